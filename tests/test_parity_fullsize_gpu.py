"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.
The oracle is evaluated on a sample of whole rows (every op is row-local, so a row of the
output depends only on the same row of x and of the residual): first/last rows of the matrix
and of tiles plus seeded random rows."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import inputs

from parity import BLOCK_FACTOR, assert_close, attention_reference, make_call, oracle_rows, run_gpu, sample_rows

pytestmark = pytest.mark.gpu
BF16 = torch.bfloat16


def announce(*a):
    print("[case]", *a, flush=True)


def test_c2_full_size_sampled_rows():
    prob = inputs.make("c2")
    announce("c2", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob, poison=True)
    assert "tile=256x256" in call.plan()
    # out was handed over full of NaN: every element must have been written (no tile skipped)
    assert torch.isfinite(got.float()).all()
    rows = sample_rows(prob.M, 64)       # at least one row of each of the 16 tile rows
    err = assert_close(got[rows], oracle_rows(prob, rows), BF16, "c2")
    print("c2 max|err| %.3e over %d rows" % (err, len(rows)))


def test_c3_full_size_sampled_rows():
    prob = inputs.make("c3")
    announce("c3", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob, poison=True)
    assert torch.isfinite(got.float()).all()      # out started as NaN: the GEMM pass staged and the finalize pass rewrote every element
    rows = sample_rows(prob.M, 64)                # at least one row of each of the 32 tile rows
    err = assert_close(got[rows], oracle_rows(prob, rows), BF16, "c3")
    print("c3 max|err| %.3e over %d rows" % (err, len(rows)))
    # LayerNorm invariant at any size: undoing the affine step leaves rows of mean 0, variance ~1
    g = prob.epilogue[2][1].double(); b = prob.epilogue[2][2].double()
    z = (got.double() - b) / g
    assert z.mean(dim=1).abs().max() < 2e-2
    assert (z.var(dim=1, unbiased=False) - 1).abs().max() < 5e-2


def test_c4_full_size_all_rows():
    prob = inputs.make("c4")
    announce("c4", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob, poison=True)
    ref = oracle_rows(prob)
    err = assert_close(got, ref, BF16, "c4")
    print("c4 max|err| %.3e, plan %s" % (err, call.plan()))
    g = got.double().numpy()
    assert np.abs(g.sum(axis=1) - 1).max() <= 4e-3                 # rows sum to one
    # the largest entry agrees up to rounding ties: the GPU's argmax is within tolerance of the true max
    idx = g.argmax(axis=1)
    top = ref.max(axis=1)
    assert np.all(ref[np.arange(ref.shape[0]), idx] >= top * (1 - 2e-2))


def test_c5_mlp_block_full_size():
    blk = inputs.make_mlp()
    T = blk.x.shape[0]
    announce("c5", T)
    p1 = blk.call1()
    h_gpu, call1 = run_gpu(p1, poison=True)
    assert torch.isfinite(h_gpu.float()).all()
    rows = sample_rows(T, 80)                     # at least one token of each of the 64 tile rows
    # call 1 against the oracle on sampled rows
    h_ref = oracle_rows(p1, rows)
    assert_close(h_gpu[rows], h_ref, BF16, "c5a")
    # end to end: GPU call 2 on the GPU's own h, oracle chain without intermediate rounding
    out_gpu, call2 = run_gpu(blk.call2(h_gpu), poison=True)
    assert torch.isfinite(out_gpu.float()).all()
    import oracle
    ep2 = [("bias",), ("residual", inputs.to_f64(blk.x[rows])),
           ("layernorm", inputs.to_f64(blk.gamma), inputs.to_f64(blk.beta), blk.eps)]
    out_ref = oracle.fused_linear_epilogue(h_ref, inputs.to_f64(blk.w2), inputs.to_f64(blk.b2), ep2)
    err = assert_close(out_gpu[rows], out_ref, BF16, "c5 end to end")
    print("c5 end-to-end max|err| %.3e; %s | %s" % (err, call1.plan(), call2.plan()))


def test_c5b_per_call_on_oracle_rounded_h():
    """Call 2 in isolation: its input h is the oracle's call-1 result rounded to bf16, fed to
    both sides; reduced to 512 tokens so that the oracle's call 1 stays within seconds."""
    blk = inputs.make_mlp()
    rows = sample_rows(blk.x.shape[0], 512, seed=3)
    xr = blk.x[rows].contiguous()
    h_in = torch.from_numpy(oracle_rows(blk.call1(xr))).to(BF16)
    p2 = blk.call2(h_in, xr)
    announce("c5b per call", p2.M, p2.N, p2.K)
    got, call = run_gpu(p2)
    sub = list(range(0, 512, 8))
    assert_close(got[sub], oracle_rows(p2, sub), BF16, "c5b " + call.plan())


def test_m1_perceptron_chain_every_layer():
    """The batch-1 perceptron of bench.py's workload m1.  Layer by layer: the GPU and the oracle both start from
    the oracle's own previous activation, rounded to the storage dtype (no oracle input comes from the GPU).
    End to end: the GPU chain on its own activations against the oracle's float64 chain."""
    ch = inputs.make_chain()
    announce("m1", len(ch.ws), ch.x.shape)
    F32 = torch.float32
    import oracle
    h_gpu, h_ref = ch.x, inputs.to_f64(ch.x)
    for i in range(len(ch.ws)):
        h_in = torch.from_numpy(h_ref).to(F32)                      # the oracle's activation as the layer's input
        prob = ch.layer(i, h_in)
        out, call = run_gpu(prob)
        assert "thin_f32" in call.plan() and "tile=8x16" in call.plan(), call.plan()
        assert_close(out, oracle_rows(prob), F32, "m1 layer %d" % i)
        h_gpu, _ = run_gpu(ch.layer(i, h_gpu))                      # the GPU's own chain
        h_ref = oracle.fused_linear_epilogue(h_ref, inputs.to_f64(ch.ws[i]), inputs.to_f64(ch.bs[i]), [("bias",), ("relu",)])
    err = assert_close(h_gpu, h_ref, F32, "m1 end to end")
    print("m1 end-to-end max|err| %.3e" % err)


def test_a1_attention_block_fullsize_sampled_tokens():
    """The attention block at the benchmark's size (16 x 2048 tokens, 2048 wide, 16 heads, causal), as bench.py
    launches it.  Checked: the first 200 tokens of two sequences in full (a causal block needs nothing after
    them)."""
    import oracle
    from paper_2511_16964_amd import binding
    announce("a1 full size")
    ap = inputs.make_attention("a1")
    B, T, C = ap.x.shape
    H, D = ap.heads, C // ap.heads
    d = lambda t: t.to("cuda:0")
    xg = d(ap.x)
    call = binding.AttentionBlockCall(xg, d(ap.w_qkv), d(ap.b_qkv), d(ap.w_o), d(ap.b_o), H, ap.causal, residual=xg)
    out = call.run()
    torch.cuda.synchronize()
    f64 = inputs.to_f64
    n_tok = 200
    for b in (0, B - 1):
        x = f64(ap.x[b:b + 1, :n_tok])
        ref = oracle.attention_block(x, f64(ap.w_qkv), f64(ap.b_qkv), f64(ap.w_o), f64(ap.b_o), H, ap.causal, residual=x)
        assert_close(out[b:b + 1, :n_tok].cpu(), ref, ap.dtype, "a1 block, sequence %d" % b, factor=BLOCK_FACTOR)


def test_a2_attention_fullsize_sampled_queries():
    """The attention kernel alone at the benchmark's size (workload a2: q, k, v of a1's shape from the seeded
    generator), as bench.py launches it: the last queries of sampled sequences and heads against all their keys
    (the oracle evaluates only those queries), and the first queries of another head."""
    import oracle
    from paper_2511_16964_amd import binding
    dt, B, T, C, H, causal = inputs.ATTENTION_SHAPES["a1"]
    D = C // H
    announce("a2 full size", B, T, H, D)
    qkv = inputs.make_qkv(0, B, T, H, D, dt)
    dev = qkv.to("cuda:0")
    got = binding.attention(dev[:, :, 0], dev[:, :, 1], dev[:, :, 2], causal)
    torch.cuda.synchronize()
    assert torch.isfinite(got.float()).all()
    f64 = inputs.to_f64
    for b, heads, first in ((3, [0, H - 1], T - 40), (B - 1, [5], T - 130)):
        sub = f64(qkv[b:b + 1][:, :, :, heads])
        ref, extra = attention_reference(sub[:, :, 0], sub[:, :, 1], sub[:, :, 2], causal, dt, first_query=first)
        assert_close(got[b:b + 1, first:][:, :, heads].cpu(), ref, dt, "a2 last queries", extra=extra)
    sub = f64(qkv[0:1, :300][:, :, :, [7]])
    ref, extra = attention_reference(sub[:, :, 0], sub[:, :, 1], sub[:, :, 2], causal, dt)
    assert_close(got[0:1, :300][:, :, [7]].cpu(), ref, dt, "a2 first queries", extra=extra)


@pytest.mark.parametrize("name,at", [("c2", 2), ("c3", 2)])
def test_full_size_with_a_store(name, at):
    """The benchmark shapes with a store put into their lists (c2: after the ReLU; c3: in front of the
    LayerNorm): out and the copy on sampled rows, and a property that holds at any size: no element of
    the copy keeps the fill, i.e. every tile wrote its part."""
    import oracle
    from parity import to_dev
    from paper_2511_16964_amd import binding
    prob = inputs.make(name)
    announce(name, "with a store at", at, prob.M, prob.N, prob.K)
    t = torch.full((prob.M, prob.N), float("nan"), dtype=prob.dtype, device="cuda:0")
    ep_cpu = list(prob.epilogue[:at]) + [("store", torch.empty(prob.M, prob.N, dtype=prob.dtype))] + list(prob.epilogue[at:])
    ep_dev = [("store", t) if e[0] == "store" else tuple(to_dev(a) if isinstance(a, torch.Tensor) else a for a in e) for e in ep_cpu]
    call = binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), ep_dev)
    out = call.run()
    torch.cuda.synchronize()
    assert "tile=256x256" in call.plan(), call.plan()
    rows = sample_rows(prob.M, 48)
    ep64 = inputs.epilogue_f64(ep_cpu, rows)
    ref = oracle.fused_linear_epilogue(inputs.to_f64(prob.x[rows]), inputs.to_f64(prob.w), inputs.to_f64(prob.b), ep64)
    assert_close(out[rows].cpu(), ref, prob.dtype, name + " out")
    assert_close(t[rows].cpu(), ep64[at][1], prob.dtype, name + " store")
    assert not bool(torch.isnan(t).any())
