"""GPU parity: the HIP path (through the C ABI) against the CPU float64 oracle, element by
element, on the same seeded inputs.  Tolerances: 1e-4 (fp32), 2e-2 (bf16); integer-valued
problems must match bit for bit."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import binding, inputs

from parity import TOL, assert_close, make_call, oracle_rows, run_gpu, sample_rows, to_dev, dev_epilogue

pytestmark = pytest.mark.gpu

F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16


def announce(*a):
    print("[case]", *a, flush=True)


# ------------------------------------------------------------------ small, complete comparisons
def test_c1_fp32_bias_gelu_erf_full():
    prob = inputs.make("c1")
    announce("c1 full", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob)
    assert "general" in call.plan()
    err = assert_close(got, oracle_rows(prob), F32, "c1")
    print("c1 max|err| %.3e" % err)


@pytest.mark.parametrize("variant,M,N,K", [
    ("tiled", 256, 256, 64), ("tiled", 300, 520, 192), ("tiled", 128, 128, 128), ("tiled", 77, 132, 64),
    ("tiled", 513, 772, 128), ("tiled", 200, 264, 72), ("tiled", 130, 132, 200), ("tiled256", 300, 520, 8), ("tiled128", 64, 128, 24),
    ("skinny", 32, 256, 64), ("skinny", 61, 132, 128), ("skinny", 7, 2052, 1024), ("skinny128", 32, 256, 256), ("skinny256", 19, 388, 512), ("skinny128", 64, 132, 384),
    ("skinny128", 64, 132, 320), ("skinny256", 40, 260, 192), ("skinny", 200, 388, 128),
    ("auto_skinny_seq", 64, 8192, 512), ("auto_skinny_seq", 33, 8196, 512), ("auto_skinny_seq", 50, 16384, 256),
    ("skinnyseq", 100, 388, 512), ("skinnyseq", 200, 260, 512), ("skinnyseq", 256, 132, 256), ("skinnyseq", 33, 132, 512), ("skinnyseq", 129, 2052, 256),
    ("general", 77, 45, 50), ("general", 33, 64, 64), ("general", 1, 1, 1),
    ("skinny_f32", 32, 256, 32), ("skinny_f32", 19, 388, 160), ("skinny128_f32", 7, 2052, 64), ("skinny256_f32", 32, 132, 384), ("skinny256_f32", 100, 260, 128),
    ("thin", 1, 16, 8), ("thin", 1, 1000, 512), ("thin", 16, 132, 264), ("thin", 17, 260, 576), ("thin", 32, 45, 520), ("thin", 5, 2052, 72), ("thin", 9, 31, 328),
])
def test_integer_inputs_are_bit_exact(variant, M, N, K):
    """Small-integer operands: every product and partial sum is exact in fp32 and the chain
    bias/relu/scale(0.5)/residual stays exactly representable in bf16, so any difference at
    all is an indexing error (tile mapping, MFMA operand layout, LDS swizzle, masking)."""
    dtype = BF16
    if variant.endswith("_f32"):   # the skinny kernel on fp32 operands
        variant, dtype = variant[:-4], F32
    prob = inputs.random_problem(11, M, N, K, dtype, ["bias", "relu", "scale", "residual"], integer=True)
    announce("integer exact", variant, dtype, M, N, K)
    seq = variant == "auto_skinny_seq"   # automatic plan: row block of 64 whose halves take turns on a 256-wide W stage
    got, call = run_gpu(prob, "auto" if seq else variant)
    if seq:
        assert "skinny" in call.plan() and "tile=64x128x256" in call.plan(), call.plan()
    ref = oracle_rows(prob)
    assert np.array_equal(ref, torch.from_numpy(ref).to(BF16).to(torch.float64).numpy()), "test premise: the exact result fits bf16"
    assert np.array_equal(got.to(torch.float64).numpy(), ref), call.plan()


@pytest.mark.parametrize("variant,split,M,N,K", [
    ("tiled128", 0, 200, 264, 100), ("tiled256", 0, 300, 520, 36), ("tiled", 0, 130, 132, 68), ("tiled128", 3, 200, 264, 200),
    ("tiled256", 2, 513, 772, 160), ("tiled256", 0, 2304, 1000, 64),
])
def test_fp32_tiled_integer_inputs_are_bit_exact(variant, split, M, N, K):
    """The fp32 tiled kernel on small-integer operands (sums far below 2^24): bit-exact, ragged K included."""
    prob = inputs.random_problem(14, M, N, K, F32, ["bias", "relu", "scale", "residual"], integer=True)
    announce("fp32 tiled integer exact", variant, split, M, N, K)
    got, call = run_gpu(prob, variant, split=split)
    assert "tiled_f32_mfma" in call.plan(), call.plan()
    rows = sample_rows(M, 128)
    assert np.array_equal(got[rows].to(torch.float64).numpy(), oracle_rows(prob, rows)), call.plan()


def test_fp32_large_shape_takes_the_tiled_kernel():
    prob = inputs.random_problem(15, 1536, 2048, 1024, F32, ["bias", "gelu_erf", "layernorm"])
    announce("fp32 tiled auto", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob)
    assert "tiled_f32_mfma" in call.plan(), call.plan()
    rows = sample_rows(prob.M, 48)
    assert_close(got[rows], oracle_rows(prob, rows), F32, call.plan())


@pytest.mark.parametrize("variant,split,dtype,M,N,K", [
    ("tiled", 0, BF16, 200, 263, 128), ("tiled256", 0, BF16, 300, 521, 72), ("tiled128", 3, BF16, 130, 133, 200), ("tiled256", 2, BF16, 513, 770, 256),
    ("tiled", 0, F32, 150, 262, 100), ("tiled256", 0, F32, 290, 515, 36), ("tiled128", 2, F32, 77, 129, 160), ("tiled", 0, BF16, 64, 1, 64),
])
def test_ragged_n_integer_inputs_are_bit_exact(variant, split, dtype, M, N, K):
    """N not a multiple of 4 (so rows of b, r and out are not vector-aligned either): the tiled kernels
    switch to their element-wise epilogue; exact on integer data, with and without a split of K."""
    prob = inputs.random_problem(16, M, N, K, dtype, ["bias", "relu", "scale", "residual"], integer=True)
    announce("ragged N integer exact", variant, split, dtype, M, N, K)
    got, call = run_gpu(prob, variant, split=split)
    assert "+edge" in call.plan(), call.plan()
    ref = oracle_rows(prob)
    assert np.array_equal(ref, torch.from_numpy(ref).to(dtype).to(torch.float64).numpy()), "test premise: the exact result fits the dtype"
    assert np.array_equal(got.to(torch.float64).numpy(), ref), call.plan()


def test_misaligned_out_and_residual_take_the_edge_epilogue():
    """N is a multiple of 4 but out and the residual start 2 bytes off a vector boundary."""
    dev = "cuda:0"
    prob = inputs.random_problem(23, 150, 264, 128, BF16, ["bias", "residual", "layernorm"])
    ref = oracle_rows(prob)
    r = prob.epilogue[1][1]
    rstore = torch.zeros((150, 264 + 8), dtype=BF16, device=dev); rstore[:, 1:265] = to_dev(r)
    ostore = torch.full((150, 264 + 8), -77.0, dtype=BF16, device=dev)
    ep = dev_epilogue(prob.epilogue); ep[1] = ("residual", rstore[:, 1:265])
    for split in (1, 2):
        ostore.fill_(-77.0)
        call = binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), ep, out=ostore[:, 1:265], variant="tiled", split=split)
        call.run(); torch.cuda.synchronize()
        assert "+edge" in call.plan(), call.plan()
        assert torch.all(ostore[:, 0] == -77.0) and torch.all(ostore[:, 265:] == -77.0)
        assert_close(ostore[:, 1:265].cpu(), ref, BF16, call.plan())


@pytest.mark.parametrize("variant,split,M,N,K", [
    ("tiled128", 0, 200, 264, 200), ("tiled256", 0, 300, 520, 72), ("tiled256", 3, 513, 772, 320), ("tiled", 0, 130, 133, 64),
    ("skinny", 0, 61, 132, 128), ("skinny256", 2, 19, 388, 512), ("skinny128", 0, 64, 132, 384), ("general", 0, 77, 45, 50), ("general", 0, 300, 264, 64),
])
def test_fp16_integer_inputs_are_bit_exact(variant, split, M, N, K):
    """fp16 operands (v_mfma_f32_32x32x16_f16 / 16x16x16_f16): exact on small integers through every kernel."""
    prob = inputs.random_problem(20, M, N, K, F16, ["bias", "relu", "scale", "residual"], integer=True)
    announce("fp16 integer exact", variant, split, M, N, K)
    got, call = run_gpu(prob, variant, split=split)
    assert "_f16_" in call.plan(), call.plan()
    ref = oracle_rows(prob)
    assert np.array_equal(ref, torch.from_numpy(ref).to(F16).to(torch.float64).numpy()), "test premise: the exact result fits fp16"
    assert np.array_equal(got.to(torch.float64).numpy(), ref), call.plan()


def test_integer_exact_on_the_256_tile():
    prob = inputs.random_problem(12, 2304, 2000, 128, BF16, ["bias", "relu", "scale", "residual"], integer=True)
    announce("integer exact 256-tile", prob.M, prob.N, prob.K)
    got, call = run_gpu(prob, "tiled256")
    assert "tile=256x256" in call.plan()
    rows = sample_rows(prob.M, 96)
    assert np.array_equal(got[rows].to(torch.float64).numpy(), oracle_rows(prob, rows))


@pytest.mark.parametrize("variant,split,M,N,K", [
    ("tiled128", 3, 200, 264, 200), ("tiled256", 5, 300, 520, 576), ("tiled", 2, 130, 132, 72), ("tiled128", 64, 77, 132, 320),
    ("tiled256", 16, 513, 772, 512), ("skinny", 4, 61, 132, 512), ("skinny256", 3, 19, 388, 768), ("skinny128", 3, 64, 132, 384),
    ("skinny128", 4, 32, 2052, 512), ("skinny", 7, 32, 260, 448), ("skinnyseq", 2, 100, 388, 512), ("skinnyseq", 3, 200, 132, 768),
])
def test_split_k_integer_inputs_are_bit_exact(variant, split, M, N, K):
    """K split over several workgroups per tile (uneven ranges, a ragged last K step, more splits
    asked for than there are K steps): the slabs and their ordered sum are exact on integer data."""
    prob = inputs.random_problem(13, M, N, K, BF16, ["bias", "relu", "scale", "residual"], integer=True)
    announce("split-K integer exact", variant, split, M, N, K)
    got, call = run_gpu(prob, variant, split=split)
    assert "split_k=1 " not in call.plan(), call.plan()
    ref = oracle_rows(prob)
    assert np.array_equal(ref, torch.from_numpy(ref).to(BF16).to(torch.float64).numpy()), "test premise: the exact result fits bf16"
    assert np.array_equal(got.to(torch.float64).numpy(), ref), call.plan()


SPLIT_SHAPES = [("skinny256", 3, 32, 2304, 1024, F32), ("tiled128", 2, 200, 392, 256), ("tiled256", 3, 150, 520, 320), ("skinny", 2, 32, 2304, 256), ("skinny128", 4, 50, 260, 1024),
                ("tiled128", 3, 200, 392, 160, F32), ("tiled128", 2, 200, 392, 256, F16), ("skinny", 2, 32, 2304, 256, F16)]


@pytest.mark.parametrize("shape", SPLIT_SHAPES, ids=lambda s: "%s-s%d-%dx%dx%d" % s[:5] + ("-" + str(s[5])[6:] if len(s) > 5 else ""))
@pytest.mark.parametrize("kinds", [[], ["bias", "gelu_erf"], ["bias", "residual", "layernorm"], ["relu", "softmax", "scale", "bias"],
                                   ["bias", "logsumexp"], ["bias", "layernorm", "gelu_tanh", "residual"]], ids=lambda k: "+".join(k) or "plain")
def test_split_k_chains(shape, kinds):
    variant, split, M, N, K = shape[:5]
    dtype = shape[5] if len(shape) > 5 else BF16
    prob = inputs.random_problem(4, M, N, K, dtype, kinds)
    announce("split-K chain", variant, split, M, N, K, dtype, kinds)
    got, call = run_gpu(prob, variant, split=split)
    assert "split_k=%d " % split in call.plan(), call.plan()
    assert_close(got, oracle_rows(prob), dtype, "%s %s" % (kinds, call.plan()))


def test_split_k_is_chosen_for_few_tiles_and_long_k():
    """Automatic plan: a problem with few output tiles and a long K is split, and agrees with the oracle."""
    for M, N, K in ((128, 1024, 4096), (48, 2048, 4096)):
        prob = inputs.random_problem(6, M, N, K, BF16, ["bias", "gelu_tanh", "layernorm"])
        announce("auto split", M, N, K)
        got, call = run_gpu(prob)
        assert "split_k=1 " not in call.plan(), call.plan()
        assert_close(got, oracle_rows(prob), BF16, call.plan())


CHAINS = [
    [], ["bias"], ["bias", "gelu_erf"], ["bias", "gelu_tanh"], ["bias", "relu", "scale", "residual"],
    ["bias", "gelu_tanh", "layernorm"], ["softmax"], ["bias", "residual", "layernorm"], ["scale", "logsumexp"],
    ["bias", "layernorm", "gelu_erf", "residual"], ["relu", "softmax", "scale", "bias"], ["bias", "logsumexp"],
]
SHAPES = [  # (variant, dtype, M, N, K): several tiles, ragged tails, both kernels and dtypes
    ("tiled", BF16, 200, 392, 128), ("tiled", BF16, 129, 260, 64), ("tiled", BF16, 150, 260, 136), ("skinny", BF16, 32, 2304, 256),
    ("skinny", BF16, 17, 392, 576), ("skinny", BF16, 50, 260, 192), ("skinny128", BF16, 40, 520, 640),
    ("skinny256", BF16, 32, 2304, 1024), ("general", BF16, 70, 97, 83),
    ("general", F32, 70, 97, 83), ("general", F32, 64, 256, 256), ("general", BF16, 37, 264, 96),
    ("tiled", F32, 200, 392, 128), ("tiled256", F32, 150, 260, 100),
    ("tiled", BF16, 129, 259, 64), ("tiled256", BF16, 150, 262, 136), ("tiled", F32, 100, 261, 96),
    ("tiled", F16, 200, 392, 128), ("tiled256", F16, 150, 262, 136), ("skinny", F16, 32, 2304, 256), ("general", F16, 70, 97, 83),
    ("auto", BF16, 48, 8192, 512), ("auto", F16, 64, 8192, 512),   # skinny kernel, one row block of 64 in two halves
    ("skinnyseq", BF16, 100, 2304, 512), ("skinnyseq", F16, 250, 520, 256),   # four and eight sub-blocks in turn
    ("skinny", F32, 32, 2304, 128), ("skinny256", F32, 17, 392, 640), ("skinny128", F32, 50, 260, 192),
    ("thin", BF16, 1, 2052, 1024), ("thin", BF16, 16, 263, 2056), ("thin", BF16, 29, 97, 520), ("thin", F16, 7, 392, 776),
    ("thin", F32, 1, 1000, 1028), ("thin", F32, 16, 261, 516), ("thin", F32, 32, 130, 2052),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "%s-%s-%dx%dx%d" % (s[0], str(s[1])[6:], s[2], s[3], s[4]))
@pytest.mark.parametrize("kinds", CHAINS, ids=lambda k: "+".join(k) or "plain")
def test_chains_small_shapes(shape, kinds):
    variant, dtype, M, N, K = shape
    prob = inputs.random_problem(3, M, N, K, dtype, kinds)
    announce("chain", variant, dtype, M, N, K, kinds)
    got, call = run_gpu(prob, variant)
    assert_close(got, oracle_rows(prob), dtype, "%s %s" % (kinds, call.plan()))


@pytest.mark.parametrize("dtype,M,N,K,tile", [
    (F32, 1, 4096, 4096, "tile=8x16"), (BF16, 1, 4096, 4096, "tile=8x16"), (F16, 3, 2048, 2048, "tile=8x16"), (F32, 8, 1000, 3000, "tile=8x16"),
    (F32, 2, 32768, 1024, "tile=8x16"), (BF16, 4, 1024, 16384, "tile=8x16"), (BF16, 1, 8192, 2048, "tile=8x16x1 "), (F32, 1, 4100, 2052, "tile=8x16x1 "), (BF16, 16, 2048, 2048, "tile=16x16"), (F16, 29, 1024, 4096, "tile=32x16"),
])
@pytest.mark.parametrize("kinds", [["bias", "relu"], ["bias", "gelu_erf", "layernorm"], ["scale", "softmax"], ["bias", "logsumexp"]], ids=lambda k: "+".join(k))
def test_perceptron_layers_take_the_thin_kernels(dtype, M, N, K, tile, kinds):
    """A few rows against a whole weight matrix (the automatic plan): the thin kernels, one launch plus
    the finalize pass of a row op, whole result against the oracle."""
    prob = inputs.random_problem(31, M, N, K, dtype, kinds)
    announce("thin auto", dtype, M, N, K, kinds)
    got, call = run_gpu(prob)
    assert "thin_" in call.plan() and tile in call.plan() and "split_k=1 " in call.plan(), call.plan()
    assert_close(got, oracle_rows(prob), dtype, call.plan())


def test_both_gelu_variants_are_distinguished_in_fp32():
    """The two GELUs differ by up to 4.7e-4, above the fp32 tolerance: a swapped variant fails."""
    prob = inputs.random_problem(5, 64, 128, 64, F32, ["scale", "gelu_tanh"])
    prob.epilogue[0] = ("scale", 3.0)
    got, _ = run_gpu(prob)
    assert_close(got, oracle_rows(prob), F32, "gelu_tanh fp32")
    swapped = inputs.Problem("x", F32, prob.x, prob.w, prob.b, [("scale", 3.0), ("gelu_erf",)])
    worst = np.abs(got.to(torch.float64).numpy() - oracle_rows(swapped)).max()
    assert worst > 2e-4


@pytest.mark.parametrize("variant,split,M,N,K", [("tiled", 0, 200, 520, 128), ("tiled256", 2, 300, 776, 256), ("skinny", 0, 32, 2304, 256),
                                                 ("general", 0, 70, 97, 83), ("tiled", 0, 150, 263, 64)])
def test_bf16_softmax_with_wide_logits(variant, split, M, N, K):
    """bf16 softmax is staged in out as the distance to the partial's maximum: logits with a spread of
    several tens (scale 16 on unit-variance sums) must still come out within the bf16 tolerance."""
    prob = inputs.random_problem(17, M, N, K, BF16, ["bias", "scale", "softmax"])
    prob.epilogue[1] = ("scale", 16.0)
    announce("wide softmax", variant, split, M, N, K)
    got, call = run_gpu(prob, variant, split=split)
    assert "staging=out" in call.plan(), call.plan()
    ref = oracle_rows(prob)
    assert ref.max() > 0.5          # peaked rows: the spread is real
    assert_close(got, ref, BF16, call.plan())
    assert np.abs(got.to(torch.float64).numpy().sum(1) - 1.0).max() < 1e-2


@pytest.mark.parametrize("variant,dtype,M,N,K", [("tiled", BF16, 200, 520, 128), ("tiled256", F16, 300, 776, 64), ("general", BF16, 70, 97, 83),
                                                 ("skinny", BF16, 32, 2304, 256), ("thin", F16, 3, 392, 520), ("thin", BF16, 20, 263, 264),
                                                 ("tiled128", BF16, 150, 392, 256), ("general", BF16, 35, 1, 54)])
def test_layernorm_of_rows_with_a_large_common_offset(variant, dtype, M, N, K):
    """A 2-byte dtype stages the values for the LayerNorm pass relative to their partial's mean: a row whose
    mean is hundreds of times its deviation (bias 100 on unit-scale sums) must still normalise correctly,
    which a plainly rounded staged value (error 0.2 .. 0.4 here) would not.  One column is the degenerate
    case: the result is beta exactly."""
    prob = inputs.random_problem(19, M, N, K, dtype, ["bias", "layernorm"])
    prob.b = torch.full_like(prob.b, 100.0)
    announce("layernorm with offset", variant, dtype, M, N, K)
    got, call = run_gpu(prob, variant, split=2 if variant == "tiled128" else 0)
    assert "staging=out" in call.plan(), call.plan()
    assert_close(got, oracle_rows(prob), dtype, call.plan())


def test_softmax_followed_by_a_residual_that_aliases_out():
    dev = "cuda:0"
    prob = inputs.random_problem(18, 150, 264, 128, BF16, ["bias", "softmax", "residual"])
    ref = oracle_rows(prob)
    out = to_dev(prob.epilogue[2][1]).clone()
    ep = dev_epilogue(prob.epilogue); ep[2] = ("residual", out)
    call = binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), ep, out=out)
    call.run(); torch.cuda.synchronize()
    assert "staging=workspace_f32" in call.plan(), call.plan()
    assert_close(out.cpu(), ref, BF16, call.plan())


def test_256_tile_row_ops_and_ragged_edges():
    for kinds in (["bias", "gelu_tanh", "layernorm"], ["softmax"], ["bias", "logsumexp"]):
        prob = inputs.random_problem(8, 2100, 2312, 128, BF16, kinds)
        announce("256-tile", kinds)
        got, call = run_gpu(prob, "tiled256")
        assert "tile=256x256" in call.plan()
        rows = sample_rows(prob.M, 64)
        assert_close(got[rows], oracle_rows(prob, rows), BF16, str(kinds))


# ------------------------------------------------------------------ edge cases
def test_empty_and_tiny():
    dev = "cuda:0"
    x = torch.zeros((0, 64), dtype=BF16, device=dev); w = torch.ones((128, 64), dtype=BF16, device=dev)
    out = binding.fused_linear_epilogue(x, w, None, [("relu",)])
    assert out.shape == (0, 128)
    # K = 0: the contraction is an empty sum
    x = torch.zeros((5, 0), dtype=F32, device=dev); w = torch.zeros((7, 0), dtype=F32, device=dev)
    b = torch.arange(7, dtype=F32, device=dev)
    out = binding.fused_linear_epilogue(x, w, b, [("bias",)])
    torch.cuda.synchronize()
    assert torch.equal(out.cpu(), torch.arange(7, dtype=F32).repeat(5, 1))
    # one row, one column
    prob = inputs.random_problem(2, 1, 1, 7, F32, ["bias", "gelu_erf"])
    got, _ = run_gpu(prob)
    assert_close(got, oracle_rows(prob), F32, "1x1")
    # N = 1 row ops: layernorm -> beta, softmax -> 1, logsumexp -> the value itself
    prob = inputs.random_problem(2, 9, 1, 16, F32, ["layernorm"])
    got, _ = run_gpu(prob)
    assert_close(got, oracle_rows(prob), F32, "ln N=1")
    prob = inputs.random_problem(2, 9, 1, 16, F32, ["softmax"])
    got, _ = run_gpu(prob)
    assert torch.equal(got, torch.ones(9, 1))


def test_strided_operands_and_in_place_residual():
    """Leading dimensions larger than the row length, and out aliasing the residual exactly."""
    dev = "cuda:0"
    prob = inputs.random_problem(21, 150, 264, 128, BF16, ["bias", "residual"])
    pad = lambda t, extra: torch.cat([t, torch.full((t.shape[0], extra), 7.0, dtype=t.dtype)], 1)
    xs = to_dev(pad(prob.x, 64))[:, :128]
    ws = to_dev(pad(prob.w, 8))[:, :128]
    r = prob.epilogue[1][1]
    rs = to_dev(pad(r, 24))[:, :264]
    ref = oracle_rows(prob)
    for variant in ("tiled", "general"):
        store = torch.empty((150, 264 + 24), dtype=BF16, device=dev)
        store[:, :264] = rs
        out_view = store[:, :264]
        got = binding.fused_linear_epilogue(xs, ws, to_dev(prob.b), [("bias",), ("residual", out_view)],
                                            out=out_view, variant=variant)
        torch.cuda.synchronize()
        assert got.data_ptr() == store.data_ptr()
        assert_close(got.cpu(), ref, BF16, "strided in-place " + variant)


def test_padding_columns_of_out_are_not_written():
    dev = "cuda:0"
    prob = inputs.random_problem(22, 140, 136, 64, BF16, ["bias", "gelu_tanh", "layernorm"])
    for variant in ("tiled", "general"):
        store = torch.full((140, 136 + 40), -77.0, dtype=BF16, device=dev)
        out_view = store[:, :136]
        binding.fused_linear_epilogue(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), dev_epilogue(prob.epilogue),
                                      out=out_view, variant=variant)
        torch.cuda.synchronize()
        assert torch.all(store[:, 136:] == -77.0)
        assert_close(out_view.cpu(), oracle_rows(prob), BF16, "padded out " + variant)


def test_results_are_bitwise_reproducible():
    prob = inputs.random_problem(9, 520, 776, 256, BF16, ["bias", "gelu_erf", "layernorm"])
    call = make_call(prob)
    first = call.run().clone()
    for _ in range(5):
        again = call.run()
        torch.cuda.synchronize()
        assert torch.equal(first, again)


def test_workspace_too_small_is_refused():
    prob = inputs.random_problem(9, 128, 256, 64, BF16, ["softmax"])
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    call = make_call(prob, workspace=small)
    with pytest.raises(binding.FleError) as e:
        call.run()
    assert e.value.status == 6


def test_structural_invariants_on_gpu():
    """Row permutation and M-splitting commute with the op (tile mapping cannot leak between rows)."""
    prob = inputs.random_problem(31, 300, 264, 128, BF16, ["bias", "gelu_tanh", "residual", "layernorm"])
    base, _ = run_gpu(prob)
    perm = torch.randperm(300, generator=torch.Generator().manual_seed(1))
    ep = list(prob.epilogue); ep[2] = ("residual", prob.epilogue[2][1][perm])
    p2 = inputs.Problem("perm", BF16, prob.x[perm], prob.w, prob.b, ep)
    got, _ = run_gpu(p2)
    assert torch.equal(got, base[perm])
    ep = list(prob.epilogue); ep[2] = ("residual", prob.epilogue[2][1][:100].contiguous())
    top, _ = run_gpu(inputs.Problem("top", BF16, prob.x[:100].contiguous(), prob.w, prob.b, ep))
    assert torch.equal(top, base[:100])


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """fle_run only launches kernels (no allocation, no synchronisation, no memset), so a sequence
    of calls can be captured once and replayed: every replay must reproduce the eager results bit
    for bit, also after the inputs have changed and with eager work between the replays."""
    dev = "cuda:0"
    probs = [inputs.random_problem(41, 64, 256, 256, F32, ["bias", "gelu_erf"]),                         # general kernel
             inputs.random_problem(42, 300, 520, 256, BF16, ["bias", "gelu_tanh", "layernorm"]),         # tiled + finalize
             inputs.random_problem(43, 48, 2048, 2048, BF16, ["softmax"]),                               # skinny, split K, staged fp32
             inputs.random_problem(44, 130, 263, 512, BF16, ["bias", "relu", "scale", "residual"])]      # edge epilogue
    calls = [make_call(p, v) for p, v in zip(probs, ("auto", "tiled", "auto", "tiled"))]
    plans = []
    for c in calls:
        c.run(); plans.append(c.plan())
    torch.cuda.synchronize()
    assert "general" in plans[0] and "tiled" in plans[1] and "skinny" in plans[2] and "split_k=1 " not in plans[2] and "+edge" in plans[3], plans
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        for c in calls:
            c.run()
    gen = torch.Generator().manual_seed(5)
    for rep in range(3):
        for c in calls:  # new x values in place: the graph reads the same buffers
            x = c._tensors[0]
            x.copy_(torch.randn(x.shape, generator=gen).to(x.dtype))
        eager = [c.run().clone() for c in calls]
        torch.cuda.synchronize()
        for c in calls:
            c.out.fill_(-5.0)
        graph.replay()
        torch.cuda.synchronize()
        for c, ref, plan in zip(calls, eager, plans):
            assert torch.equal(c.out, ref), "replay %d differs: %s" % (rep, plan)
    # the last replay also agrees with the oracle on the current inputs
    for c, p in zip(calls, probs):
        cur = inputs.Problem("cur", p.dtype, c._tensors[0].cpu(), p.w, p.b, p.epilogue)
        assert_close(c.out.cpu(), oracle_rows(cur), p.dtype, "graph replay vs oracle")


@pytest.mark.parametrize("variant,M,N,K,kinds", [
    ("skinny", 8, 33024, 64, ["softmax"]), ("skinny", 8, 33024, 64, ["bias", "logsumexp"]),     # 1032 partials per row
    ("tiled128", 40, 4352, 64, ["bias", "gelu_tanh", "layernorm"]),                              # 68 LayerNorm partials per row
    ("general", 5, 1100, 32, ["layernorm"]), ("general", 5, 17000, 16, ["softmax"]),            # 69 and 1063 partials
])
def test_rows_with_many_partials(variant, M, N, K, kinds):
    """Rows whose partial statistics do not fit one lane each (LayerNorm: more than 64; softmax: more
    than 1024, which leaves the register-resident batch)."""
    prob = inputs.random_problem(19, M, N, K, BF16, kinds)
    announce("many partials", variant, M, N, K, kinds)
    got, call = run_gpu(prob, variant)
    assert_close(got, oracle_rows(prob), BF16, call.plan())


def test_calls_on_side_streams_run_concurrently_and_independently():
    """Two calls with their own workspaces, enqueued on two side streams (default priority), interleaved
    several times: each must equal its result on the default stream, bit for bit."""
    pa = inputs.random_problem(51, 300, 1032, 512, BF16, ["bias", "gelu_tanh", "layernorm"])
    pb = inputs.random_problem(52, 48, 2048, 2048, BF16, ["softmax"])
    ca, cb = make_call(pa), make_call(pb)
    ra, rb = ca.run().clone(), cb.run().clone()
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(5):
        ca.out.fill_(0); cb.out.fill_(0)
        torch.cuda.synchronize()
        ca.run(stream=sa); cb.run(stream=sb); ca.run(stream=sa); cb.run(stream=sb)
        sa.synchronize(); sb.synchronize()
        assert torch.equal(ca.out, ra) and torch.equal(cb.out, rb)
