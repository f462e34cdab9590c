"""GPU parity of the grouped form (rows cut into groups, one weight matrix per group, one launch)
against the CPU oracle's loop over groups.  Same bars as the plain form: integer-valued problems
bit for bit, floating point within 1e-4 (fp32), 2e-2 (bf16), 4e-3 (fp16)."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import binding, inputs

from parity import assert_close, oracle_grouped, oracle_rows, run_gpu, run_grouped_gpu, sample_rows

pytestmark = pytest.mark.gpu

F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16


def announce(*a):
    print("[case]", *a, flush=True)


@pytest.mark.parametrize("variant,counts,N,K", [
    ("tiled128", [128, 128], 128, 64),                       # whole tiles
    ("tiled128", [1, 0, 130, 127, 0, 0, 300, 5], 264, 128),   # ragged groups, empty groups, ragged N tiles
    ("tiled256", [256, 1, 255, 257, 0, 513], 520, 72),        # ragged K step
    ("tiled256", [40], 256, 64),                              # one group
    ("tiled128", [0, 0, 77], 132, 192),                       # leading empty groups
    ("tiled128", [3] * 150, 132, 64),                         # more than 64 groups (several passes of the group scan)
    ("tiled256", [0] * 70 + [300, 20] + [0] * 60 + [1], 260, 64),
    ("auto", [50, 60, 70, 80], 1024, 256),
])
def test_grouped_integer_inputs_are_bit_exact(variant, counts, N, K):
    """Small-integer operands make every value exact, so any difference is an indexing error: the
    tile -> group mapping, a group's row limit, its W or bias pointer."""
    gp = inputs.random_grouped(21, counts, N, K, BF16, ["bias", "relu", "scale", "residual"], integer=True)
    announce("grouped integer exact", variant, len(counts), gp.M, N, K)
    got, call = run_grouped_gpu(gp, variant)
    assert "grouped_tiled_bf16_mfma" in call.plan(), call.plan()
    ref = oracle_grouped(gp)
    assert np.array_equal(ref, torch.from_numpy(ref).to(BF16).to(torch.float64).numpy()), "test premise: the exact result fits bf16"
    assert np.array_equal(got.to(torch.float64).numpy(), ref), call.plan()


@pytest.mark.parametrize("dtype,variant,counts,N,K", [
    (F32, "tiled128", [100, 0, 200, 33], 264, 100), (F32, "tiled256", [300, 10, 290], 520, 36),
    (F16, "tiled128", [100, 0, 200, 33], 264, 128), (F16, "tiled256", [300, 10, 290], 520, 72),
])
def test_grouped_other_dtypes_integer_exact(dtype, variant, counts, N, K):
    gp = inputs.random_grouped(22, counts, N, K, dtype, ["bias", "relu", "scale", "residual"], integer=True)
    announce("grouped integer exact", dtype, variant, gp.M, N, K)
    got, call = run_grouped_gpu(gp, variant)
    assert np.array_equal(got.to(torch.float64).numpy(), oracle_grouped(gp)), call.plan()


CHAINS = [
    ["softmax", "bias"],                       # a bias after the row op: the finalize pass must pick the row's group
    ["bias", "layernorm", "bias", "relu"],
    ["bias", "gelu_tanh"],
    ["bias", "gelu_erf", "scale", "residual"],
    ["bias", "relu", "layernorm", "residual"],
    ["scale", "softmax"],
    ["bias", "residual", "logsumexp"],
    [],
]


@pytest.mark.parametrize("kinds", CHAINS, ids=lambda k: "+".join(k) or "none")
@pytest.mark.parametrize("dtype,variant,counts,N,K", [
    (BF16, "tiled128", [70, 0, 200, 129, 1], 392, 256),
    (BF16, "tiled256", [300, 260, 5, 0, 255], 772, 192),
    (F16, "auto", [64, 64, 100], 260, 128),
    (F32, "auto", [90, 10, 150], 264, 64),
])
def test_grouped_chains_match_oracle(dtype, variant, counts, N, K, kinds):
    gp = inputs.random_grouped(23, counts, N, K, dtype, kinds)
    announce("grouped chain", dtype, variant, gp.M, N, K, kinds)
    got, call = run_grouped_gpu(gp, variant)
    assert_close(got, oracle_grouped(gp), dtype, call.plan())


@pytest.mark.parametrize("N,b_shared,kinds", [
    (263, False, ["bias", "gelu_tanh", "residual"]),    # ragged N: element-wise epilogue
    (263, False, ["bias", "softmax"]),
    (264, True, ["bias", "relu"]),                       # one bias for all groups
    (130, False, ["bias", "scale", "layernorm"]),        # bias stride 130: 4-column groups break
])
def test_grouped_edge_epilogue_and_bias_layouts(N, b_shared, kinds):
    gp = inputs.random_grouped(24, [120, 0, 140, 3, 260], N, 128, BF16, kinds, shared_bias=b_shared)
    announce("grouped edge", N, b_shared, kinds)
    got, call = run_grouped_gpu(gp)
    assert ("+edge" in call.plan()) == (N % 4 != 0), call.plan()
    assert_close(got, oracle_grouped(gp), BF16, call.plan())


def test_one_group_equals_the_plain_call_bitwise():
    """G = 1 runs the same tiles in the same order as the plain tiled kernel: identical bits."""
    gp = inputs.random_grouped(25, [700], 520, 256, BF16, ["bias", "gelu_erf", "residual"])
    plain = inputs.Problem("p", BF16, gp.x, gp.w[0], gp.b[0], gp.epilogue)
    for variant in ("tiled128", "tiled256"):
        announce("grouped G=1 vs plain", variant)
        a, call = run_grouped_gpu(gp, variant)
        b, _ = run_gpu(plain, variant)
        assert torch.equal(a, b), call.plan()


def test_equal_weights_in_every_group_equal_the_plain_result():
    gp = inputs.random_grouped(26, [100, 28, 128, 300], 384, 128, BF16, ["bias", "relu", "scale"])
    gp.w = gp.w[:1].expand(4, -1, -1).contiguous()
    gp.b = gp.b[:1].expand(4, -1).contiguous()
    plain = inputs.Problem("p", BF16, gp.x, gp.w[0], gp.b[0], gp.epilogue)
    announce("grouped equal weights")
    got, call = run_grouped_gpu(gp, "tiled128")
    assert_close(got, oracle_rows(plain), BF16, call.plan())


def test_malformed_offsets_stay_in_bounds_and_cover_what_they_can():
    """Offsets beyond M or decreasing are clamped by the kernel: rows that a (clamped) group owns
    are computed with that group's weights, the rest of out is left as it was."""
    gp = inputs.random_grouped(27, [100, 100, 100], 264, 128, BF16, ["bias", "relu", "scale", "residual"], integer=True)
    ref = oracle_grouped(gp)
    announce("grouped malformed offsets")
    canary = torch.full((gp.M, gp.N), 77.0, dtype=BF16, device="cuda:0")
    # group 0: rows 0..99; group 1: [100, 5000) clamps to 100..299; group 2: (5000 -> 300, -7 -> 300): empty
    got, call = run_grouped_gpu(gp, "tiled128", offsets=[0, 100, 5000, -7], shared_out=canary)
    ref2 = inputs.GroupedProblem(gp.dtype, gp.x, gp.w[:2], gp.b[:2], [0, 100, 300], gp.epilogue)
    assert np.array_equal(got.to(torch.float64).numpy(), oracle_grouped(ref2)), call.plan()
    # rows 200..299 unowned: untouched
    canary.fill_(77.0)
    got, _ = run_grouped_gpu(gp, "tiled128", offsets=[0, 100, 200, 200], shared_out=canary)
    assert np.array_equal(got[:200].to(torch.float64).numpy(), ref[:200])
    assert (got[200:] == 77.0).all()


def test_grouped_offsets_written_by_a_kernel_on_the_same_stream():
    """The library reads the offsets on the device only: they may come from a kernel that is still
    queued when the call is made (a router), with no host synchronisation in between."""
    counts = [150, 0, 90, 272]
    gp = inputs.random_grouped(28, counts, 392, 128, BF16, ["bias", "gelu_tanh"])
    announce("grouped device-side offsets")
    dev = "cuda:0"
    cnt = torch.tensor(counts, dtype=torch.int64, device=dev)
    off = torch.zeros(len(counts) + 1, dtype=torch.int64, device=dev)
    x, w, b = gp.x.to(dev), gp.w.to(dev), gp.b.to(dev)
    torch.cuda.synchronize()
    off[1:] = torch.cumsum(cnt, 0)                    # queued, not awaited
    out = binding.grouped_fused_linear_epilogue(x, w, b, off, gp.epilogue)
    torch.cuda.synchronize()
    assert_close(out.cpu(), oracle_grouped(gp), BF16, "device offsets")


def test_grouped_routed_batch_sampled_rows():
    """A routed batch at a realistic shape (32 groups, skewed sizes with empty groups), checked on
    sampled rows that include every group's first and last row."""
    counts = inputs.routed_counts(5, 8192, 32, skew=0.3)
    gp = inputs.random_grouped(29, counts, 2048, 1024, BF16, ["bias", "gelu_tanh"])
    announce("grouped routed", gp.M, gp.N, gp.K, counts)
    got, call = run_grouped_gpu(gp)
    rows = set(sample_rows(gp.M, 40))
    for lo, hi in zip(gp.offsets, gp.offsets[1:]):
        if hi > lo:
            rows.update((lo, hi - 1))
    rows = sorted(rows)
    assert_close(got[rows], oracle_grouped(gp, rows), BF16, call.plan())


@pytest.mark.parametrize("name,tile", [("g1", "tile=256x256"), ("g2", "tile=128x128")])
def test_grouped_benchmark_workloads_full_size_sampled_rows(name, tile):
    """The grouped benchmark workloads at full size, in the launch configuration bench.py times:
    sampled rows (every group's first and last row, tile boundaries, random rows) against the oracle,
    and a poison check that every row of out was written."""
    gp = inputs.make_grouped(name)
    announce(name, gp.M, gp.N, gp.K, len(gp.offsets) - 1)
    poison = torch.full((gp.M, gp.N), float("nan"), dtype=BF16, device="cuda:0")
    got, call = run_grouped_gpu(gp, shared_out=poison)
    assert tile in call.plan() and "grouped" in call.plan(), call.plan()
    assert torch.isfinite(got.float()).all()
    rows = set(sample_rows(gp.M, 24, tile=1024 if gp.M > 8192 else 256))   # (g1: one row of every 1024; the groups' edges follow)
    for lo, hi in zip(gp.offsets, gp.offsets[1:]):
        if hi > lo:
            rows.update((lo, hi - 1))
    rows = sorted(rows)
    err = assert_close(got[rows], oracle_grouped(gp, rows), BF16, call.plan())
    print("%s max|err| %.3e over %d rows" % (name, err, len(rows)))
