"""GPU parity of the attention kernel and of the three-launch attention block against the CPU oracle
(scaled dot-product attention written out in float64).  Floating point within 2e-2 (bf16) / 4e-3 (fp16)
of the oracle, the same criterion as the fused linear operator; the block, with its two stored intermediates,
gets sqrt(3) times that allowance (three roundings in sequence)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_16964_amd import binding, inputs

from parity import BLOCK_FACTOR, assert_close, attention_reference

pytestmark = pytest.mark.gpu

BF16, F16 = torch.bfloat16, torch.float16
DEV = "cuda:0"


def announce(*a):
    print("[case]", *a, flush=True)


def run_attention(qkv, causal, scale=None):
    d = qkv.to(DEV)
    out = binding.attention(d[:, :, 0], d[:, :, 1], d[:, :, 2], causal, scale)
    torch.cuda.synchronize()
    return out.cpu()


def check_attention(got, qkv, causal, dtype, what="", scale=None):
    """got against the oracle on the packed [B,T,3,H,D] operands, under the attention kernel's criterion."""
    f = inputs.to_f64(qkv)
    ref, extra = attention_reference(f[:, :, 0], f[:, :, 1], f[:, :, 2], causal, dtype, scale)
    assert_close(got, ref, dtype, what, extra=extra)


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("D", [32, 64, 128, 256])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("T", [1, 2, 31, 64, 65, 128, 129, 200, 257, 333])
def test_attention_small(dtype, D, causal, T):
    """One to three workgroups per head along the queries, ragged key blocks, several heads and batches."""
    announce("attention small", dtype, D, causal, T)
    qkv = inputs.make_qkv(100 + T, 2, T, 3, D, dtype)
    check_attention(run_attention(qkv, causal), qkv, causal, dtype, "T=%d" % T)


@pytest.mark.parametrize("dtype,D,causal,B,H,T", [
    (BF16, 128, True, 8, 32, 300),    # hundreds of heads: several rounds of workgroups per XCD, ragged last query block
    (BF16, 64, False, 4, 64, 520),
    (F16, 128, False, 16, 16, 513),
    (F16, 64, True, 2, 128, 777),
    (BF16, 64, True, 3, 7, 400),      # a head count that is not a multiple of 8 (plain work order)
    (BF16, 128, True, 1, 24, 1100),   # 3 heads per XCD, fewer than a head group
    (BF16, 64, False, 5, 16, 260),    # 10 heads per XCD: a full group of 8 and a rest of 2
    (BF16, 32, True, 4, 24, 600),     # head dimension 32: a K / V row is a quarter of a bank sweep
    (F16, 256, True, 2, 16, 700),     # head dimension 256: one workgroup per CU
])
def test_attention_many_heads(dtype, D, causal, B, H, T):
    announce("attention wide", dtype, D, causal, B, H, T)
    qkv = inputs.make_qkv(7, B, T, H, D, dtype)
    check_attention(run_attention(qkv, causal), qkv, causal, dtype)


@pytest.mark.parametrize("dtype,D,T,G", [
    (BF16, 128, 300, 7), (BF16, 64, 300, 64), (F16, 128, 513, 100), (BF16, 128, 257, 128), (F16, 64, 200, 2),
    (BF16, 64, 130, 129), (BF16, 128, 130, 1000),       # a group that holds (nearly) the whole sequence
])
def test_attention_group_causal(dtype, D, T, G):
    """Causal over groups of G tokens: group edges inside, at and across the 64-key blocks and 128-query blocks."""
    announce("attention group causal", dtype, D, T, G)
    qkv = inputs.make_qkv(300 + G, 2, T, 3, D, dtype)
    check_attention(run_attention(qkv, G), qkv, G, dtype, "G=%d" % G)


@pytest.mark.parametrize("dtype,D,T,Tk,causal", [
    (BF16, 64, 77, 300, 0),       # cross attention: fewer queries than keys, no mask
    (BF16, 128, 300, 77, 0),      # more queries than keys
    (F16, 64, 100, 356, 1),       # causal continuation: 100 new tokens after 256 kept keys
    (BF16, 128, 1, 500, 1),       # one new token
    (BF16, 32, 130, 400, 64),     # groups of 64 tokens, the queries start inside a group
    (F16, 256, 200, 201, 1),
])
def test_attention_with_different_query_and_key_counts(dtype, D, T, Tk, causal):
    announce("attention Tq != Tk", dtype, D, T, Tk, causal)
    B, H = 2, 3
    q = inputs.make_qkv(900 + T, B, T, H, D, dtype)[:, :, 0]
    kv = inputs.make_qkv(901 + Tk, B, Tk, H, D, dtype)
    d = lambda t: t.to(DEV)
    got = binding.attention(d(q), d(kv)[:, :, 1], d(kv)[:, :, 2], causal)
    torch.cuda.synchronize()
    f = inputs.to_f64
    ref, extra = attention_reference(f(q), f(kv[:, :, 1]), f(kv[:, :, 2]), causal, dtype)
    assert_close(got.cpu(), ref, dtype, extra=extra)


def test_attention_on_sequence_first_tensors():
    """[T, B, ...] tensors (the layout of sequence-first modules) viewed as [B, T, H, D]: the token stride is
    B rows, the sequence stride one row; input and output are used in place."""
    announce("attention sequence-first")
    T, B, H, D = 150, 3, 2, 64
    qkv = inputs.make_qkv(33, B, T, H, D, BF16)                       # [B,T,3,H,D], the values to use
    tb = qkv.transpose(0, 1).contiguous().to(DEV)                     # [T,B,3,H,D] in memory
    q, k, v = (tb[:, :, i].transpose(0, 1) for i in range(3))         # [B,T,H,D] views
    out_tb = torch.zeros(T, B, H, D, device=DEV, dtype=BF16)
    binding.attention(q, k, v, True, out=out_tb.transpose(0, 1))
    torch.cuda.synchronize()
    check_attention(out_tb.transpose(0, 1).cpu(), qkv, True, BF16)


@pytest.mark.parametrize("causal", [0, 1, 1000])
def test_attention_long_sequence_sampled_queries(causal):
    """40 000 tokens in one sequence (625 key blocks, 313 query blocks): the first and the last queries against the
    oracle, which evaluates only those."""
    announce("attention long sequence", causal)
    B, T, H, D = 1, 40000, 2, 64
    qkv = inputs.make_qkv(77, B, T, H, D, BF16)
    got = run_attention(qkv, causal)
    assert torch.isfinite(got.float()).all()
    f = inputs.to_f64(qkv)
    tail, extra = attention_reference(f[:, :, 0], f[:, :, 1], f[:, :, 2], causal, BF16, first_query=T - 6)
    assert_close(got[:, T - 6:], tail, BF16, "last queries", extra=extra)
    if causal:   # the first queries only see the first keys: a short problem of its own
        n = 2100 if causal == 1 else 2000     # with groups of 1000 tokens, queries 0 .. 1999 see exactly keys 0 .. 1999
        head, extra = attention_reference(f[:, :n, 0], f[:, :n, 1], f[:, :n, 2], causal, BF16)
        assert_close(got[:, :n], head, BF16, "first queries", extra=extra)


def test_attention_peaked_and_flat_scores():
    """Score spreads far from the N(0,1) of the workload: nearly one-hot rows (large scale) and nearly
    uniform rows (tiny scale); the running maximum must keep both finite."""
    for spread, scale in ((4.0, None), (1.0, 1e-3), (1.0, 2.0)):
        announce("attention spread", spread, scale)
        qkv = inputs.make_qkv(11, 2, 190, 2, 64, BF16, spread)
        got = run_attention(qkv, True, scale)
        assert torch.isfinite(got.float()).all()
        check_attention(got, qkv, True, BF16, scale=scale)


def test_attention_separate_tensors_and_out():
    """q, k, v as three separate packed tensors, result written into a strided view."""
    announce("attention separate operands")
    B, T, H, D = 2, 150, 2, 128
    qkv = inputs.make_qkv(3, B, T, H, D, BF16)
    q, k, v = (qkv[:, :, i].contiguous().to(DEV) for i in range(3))
    buf = torch.zeros(B, T, 2, H, D, device=DEV, dtype=BF16)
    binding.attention(q, k, v, False, out=buf[:, :, 1])
    torch.cuda.synchronize()
    check_attention(buf[:, :, 1].cpu(), qkv, False, BF16)
    assert (buf[:, :, 0] == 0).all()


def test_attention_rejects_what_it_cannot_run():
    qkv = inputs.make_qkv(1, 1, 8, 1, 64, BF16).to(DEV)
    q, k, v = qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2]
    with pytest.raises(binding.FleError):
        binding.attention(q.float(), k.float(), v.float(), False)          # fp32
    bad = inputs.make_qkv(1, 1, 8, 1, 16, BF16).to(DEV)
    with pytest.raises(binding.FleError):
        binding.attention(bad[:, :, 0], bad[:, :, 1], bad[:, :, 2], False)  # head dimension 16
    with pytest.raises(binding.FleError):
        binding.attention(q, k, v, False, scale=-1.0)
    with pytest.raises(binding.FleError):
        binding.attention(q, k, v, -3)                                     # negative group size
    with pytest.raises(binding.FleError):
        binding.attention(q, k[:, :4], v[:, :4], True)                     # causal with fewer keys than queries
    with pytest.raises(binding.FleError):
        binding.attention(q, k, v, False, out=q)                           # o overlaps q


def run_block(ap):
    d = lambda t: None if t is None else t.to(DEV)
    x = d(ap.x)
    out = binding.attention_block(x, d(ap.w_qkv), d(ap.b_qkv), d(ap.w_o), d(ap.b_o), ap.heads, ap.causal,
                                  residual=x if ap.residual is not None else None)
    torch.cuda.synchronize()
    return out.cpu()


def oracle_block(ap):
    f = inputs.to_f64
    return oracle.attention_block(f(ap.x), f(ap.w_qkv), f(ap.b_qkv), f(ap.w_o), f(ap.b_o), ap.heads, ap.causal,
                                  residual=f(ap.residual))


@pytest.mark.parametrize("dtype,B,T,C,heads,causal,bias,residual", [
    (BF16, 2, 200, 256, 2, True, True, True),
    (BF16, 3, 77, 512, 8, False, True, False),
    (F16, 2, 130, 384, 3, True, False, True),
    (BF16, 1, 1, 128, 2, True, True, True),
    (BF16, 2, 150, 256, 8, True, True, True),     # head dimension 32
    (F16, 1, 260, 512, 2, False, True, False),    # head dimension 256
])
def test_attention_block_small(dtype, B, T, C, heads, causal, bias, residual):
    announce("attention block", dtype, B, T, C, heads, causal, bias, residual)
    ap = inputs.make_attention("a1", 5, B=B, T=T, C=C, heads=heads, causal=causal, dtype=dtype, bias=bias, residual=residual)
    assert_close(run_block(ap), oracle_block(ap), dtype, factor=BLOCK_FACTOR)


def test_attention_block_in_place():
    """out == residual == x: the block overwrites its input (x is last read by the first stage)."""
    announce("attention block in place")
    ap = inputs.make_attention("a1", 9, B=2, T=140, C=256, heads=4, causal=True, dtype=BF16)
    d = lambda t: t.to(DEV)
    x = d(ap.x).clone()
    out = binding.attention_block(x, d(ap.w_qkv), d(ap.b_qkv), d(ap.w_o), d(ap.b_o), ap.heads, ap.causal, residual=x, out=x)
    torch.cuda.synchronize()
    assert out.data_ptr() == x.data_ptr()
    assert_close(x.cpu(), oracle_block(ap), BF16, factor=BLOCK_FACTOR)
    other = torch.empty_like(x)
    with pytest.raises(binding.FleError):   # out on top of x without being the residual
        binding.attention_block(x, d(ap.w_qkv), d(ap.b_qkv), d(ap.w_o), d(ap.b_o), ap.heads, ap.causal, residual=other, out=x)


def test_attention_block_in_a_hip_graph():
    """The block only launches kernels (no allocation, synchronisation or memset), so its three stages can be
    captured once and replayed; every replay reproduces the eager result bit for bit on changed inputs."""
    announce("attention block in a graph")
    ap = inputs.make_attention("a1", 21, B=2, T=300, C=256, heads=2, causal=True, dtype=BF16)
    d = lambda t: t.to(DEV)
    x = d(ap.x)
    call = binding.AttentionBlockCall(x, d(ap.w_qkv), d(ap.b_qkv), d(ap.w_o), d(ap.b_o), ap.heads, ap.causal, residual=x)
    call.run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        call.run()
    gen = torch.Generator().manual_seed(3)
    for rep in range(3):
        x.copy_(torch.randn(x.shape, generator=gen).to(x.dtype))
        eager = call.run().clone()
        torch.cuda.synchronize()
        call.out.fill_(-5.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(call.out, eager), "replay %d differs" % rep
    cur = inputs.AttentionProblem("cur", BF16, ap.heads, ap.causal, x.cpu(), ap.w_qkv, ap.b_qkv, ap.w_o, ap.b_o, x.cpu())
    assert_close(call.out.cpu(), oracle_block(cur), BF16, factor=BLOCK_FACTOR)
