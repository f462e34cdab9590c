"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.
The oracle is evaluated on a sample of whole rows (every op is row-local, so a row of the
output depends only on the same row of x and of the residual): first/last rows of the matrix
and of tiles plus seeded random rows."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import inputs

from parity import BLOCK_FACTOR, assert_close, value_scale, make_call, oracle_rows, run_gpu, sample_rows

pytestmark = pytest.mark.gpu
BF16 = torch.bfloat16


def announce(*a):
    print("[case]", *a, flush=True)


def test_c2_full_size_sampled_rows():
    prob = inputs.make("c2")
    announce("c2", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob)
    assert "tile=256x256" in call.plan()
    rows = sample_rows(prob.M, 64)
    err = assert_close(got[rows], oracle_rows(prob, rows), BF16, "c2")
    print("c2 max|err| %.3e over %d rows" % (err, len(rows)))
    # every output element is finite and no tile was skipped (poison check)
    assert torch.isfinite(got.float()).all()


def test_c3_full_size_sampled_rows():
    prob = inputs.make("c3")
    announce("c3", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob)
    rows = sample_rows(prob.M, 64)
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
    got, call = run_gpu(prob)
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
    h_gpu, call1 = run_gpu(p1)
    rows = sample_rows(T, 48)
    # call 1 against the oracle on sampled rows
    h_ref = oracle_rows(p1, rows)
    assert_close(h_gpu[rows], h_ref, BF16, "c5a")
    # end to end: GPU call 2 on the GPU's own h, oracle chain without intermediate rounding
    out_gpu, call2 = run_gpu(blk.call2(h_gpu))
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
    """The batch-1 perceptron of bench.py's workload m1: every layer's GPU output against the oracle applied
    to the same input (the GPU's own previous activation), and the chain end to end against the oracle's
    float64 chain."""
    ch = inputs.make_chain()
    announce("m1", len(ch.ws), ch.x.shape)
    F32 = torch.float32
    h_gpu, h_ref = ch.x, inputs.to_f64(ch.x)
    import oracle
    for i in range(len(ch.ws)):
        prob = ch.layer(i, h_gpu)
        out, call = run_gpu(prob)
        assert "thin_f32" in call.plan() and "tile=8x16" in call.plan(), call.plan()
        assert_close(out, oracle_rows(prob), F32, "m1 layer %d" % i)
        h_ref = oracle.fused_linear_epilogue(h_ref, inputs.to_f64(ch.ws[i]), inputs.to_f64(ch.bs[i]), [("bias",), ("relu",)])
        h_gpu = out
    err = assert_close(h_gpu, h_ref, F32, "m1 end to end")
    print("m1 end-to-end max|err| %.3e" % err)


def test_a1_attention_block_fullsize_sampled_tokens():
    """The attention block at the benchmark's size (16 x 2048 tokens, 2048 wide, 16 heads, causal), as bench.py
    launches it.  Checked: the first 200 tokens of two sequences in full (a causal block needs nothing after
    them), and late tokens of one sequence and head through the attention kernel alone (the oracle evaluates
    only the sampled queries, against all their keys)."""
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
    # the attention kernel on the block's own qkv (left in the workspace by the run above): last queries of a sequence
    ws = call._keep[-1]
    qkv = ws[:B * T * 3 * C * 2].view(ap.dtype).view(B, T, 3, H, D)
    b, heads, first = 3, [0, H - 1], T - 40
    got = binding.attention(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], True)
    torch.cuda.synchronize()
    sub = f64(qkv[b:b + 1][:, :, :, heads].cpu())
    ref = oracle.attention(sub[:, :, 0], sub[:, :, 1], sub[:, :, 2], True, first_query=first)
    assert_close(got[b:b + 1, first:][:, :, heads].cpu(), ref, ap.dtype, "a1 attention, last queries", s=value_scale(qkv[:, :, 2]))
