"""GPU parity of a LayerNorm of x over K in front of the multiplication (normalisation -> projection): inside the
dot-product kernel's own sweep for a few rows of x, as a pass into the workspace in front of every other kernel.  The
oracle normalises the stored x in float64 (definition pinned on the CPU side) and multiplies the unrounded result."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import binding, inputs

from parity import assert_close, oracle_rows, run_gpu, sample_rows

pytestmark = pytest.mark.gpu

F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16


def announce(*a):
    print("[case]", *a, flush=True)


@pytest.mark.parametrize("dtype,M", [(BF16, 1), (BF16, 2), (BF16, 3), (BF16, 4), (F16, 1), (F16, 4), (F32, 1), (F32, 3), (F32, 4)])
@pytest.mark.parametrize("N,K", [(1024, 1024), (4096, 4096), (520, 2048), (4100, 4104)])
@pytest.mark.parametrize("kinds", [["bias", "gelu_erf"], ["bias", "relu", "layernorm"]])
def test_few_rows_normalise_inside_the_dot_product_kernel(dtype, M, N, K, kinds):
    prob = inputs.random_problem(61, M, N, K, dtype, kinds, ln_pre=True)
    announce("ln_pre fused", dtype, M, N, K, kinds)
    got, call = run_gpu(prob, "thin", poison=True)
    assert "ln_pre=fused" in call.plan() and "_dot" in call.plan(), call.plan()
    assert_close(got, oracle_rows(prob), dtype, what="ln_pre fused %s" % call.plan())


@pytest.mark.parametrize("dtype", [BF16, F32])
def test_fused_form_without_gamma_or_beta_and_off_centre_rows(dtype):
    """gamma / beta absent (1 / 0), and rows whose mean is 30 deviations from zero (the kernel's one-sweep variance
    is E[x^2] - mean^2 in fp32)."""
    for g_on, b_on, x_mean in ((False, True, 0.5), (True, False, 0.5), (False, False, 0.5), (True, True, 30.0)):
        prob = inputs.random_problem(63, 2, 2048, 4096, dtype, ["bias"], ln_pre=True, x_mean=x_mean)
        e = prob.epilogue[0]
        prob.epilogue[0] = ("layernorm_pre", e[1] if g_on else None, e[2] if b_on else None, e[3])
        announce("ln_pre fused", dtype, g_on, b_on, x_mean)
        got, call = run_gpu(prob, "thin", poison=True)
        assert "ln_pre=fused" in call.plan()
        assert_close(got, oracle_rows(prob), dtype, what="ln_pre fused gamma %s beta %s mean %s" % (g_on, b_on, x_mean))


@pytest.mark.parametrize("dtype,variant,M,N,K", [
    (BF16, "auto", 300, 520, 512), (BF16, "tiled256", 513, 772, 1024), (BF16, "tiled128", 77, 132, 128), (BF16, "skinny256", 64, 4096, 1024),
    (BF16, "thin", 16, 1024, 2048), (BF16, "general", 33, 70, 100), (F16, "auto", 130, 260, 200), (F32, "auto", 130, 260, 203),
    (F32, "tiled128", 200, 264, 512), (BF16, "auto", 1000, 132, 147), (BF16, "auto", 2, 64, 64), (F32, "thin", 8, 4096, 4096), (F32, "thin", 5, 1024, 2048),
])
@pytest.mark.parametrize("kinds", [["bias", "gelu_tanh"], ["bias", "residual", "layernorm"], ["scale", "softmax"]])
def test_other_shapes_normalise_in_a_pass_of_their_own(dtype, variant, M, N, K, kinds):
    prob = inputs.random_problem(67, M, N, K, dtype, kinds, ln_pre=True)
    announce("ln_pre pass", dtype, variant, M, N, K, kinds)
    got, call = run_gpu(prob, variant, poison=True)
    assert "ln_pre=pass" in call.plan(), call.plan()
    assert_close(got, oracle_rows(prob), dtype, what="ln_pre pass %s" % call.plan())


def test_misaligned_x_rows_still_reach_the_fast_kernels():
    """The normalised copy is contiguous and aligned whatever x looks like: x with an odd leading dimension and a
    2-byte offset takes the tiled kernel after the pass (alone it would fall to the general kernel)."""
    prob = inputs.random_problem(69, 1024, 1024, 1024, BF16, ["bias", "relu"], ln_pre=True)
    dev = "cuda:0"
    buf = torch.zeros(1024, 1024 + 3, dtype=BF16, device=dev)
    xv = buf[:, 1:1025]
    xv.copy_(prob.x.to(dev))
    ep = [tuple(t.to(dev) if isinstance(t, torch.Tensor) else t for t in e) for e in prob.epilogue]
    call = binding.Call(xv, prob.w.to(dev), prob.b.to(dev), ep)
    got = call.run().cpu()
    assert "tiled" in call.plan() and "ln_pre=pass" in call.plan(), call.plan()
    assert_close(got, oracle_rows(prob), BF16, what="misaligned x")
    plain = binding.Call(xv, prob.w.to(dev), prob.b.to(dev), ep[1:])
    assert "general" in plain.plan()


def test_full_size_projection_behind_a_layernorm():
    """A transformer block's normalisation -> projection at benchmark size (4096 tokens, 4096 -> 4096), sampled rows."""
    prob = inputs.random_problem(71, 4096, 4096, 4096, BF16, ["bias", "gelu_erf"], ln_pre=True)
    announce("ln_pre full size")
    got, call = run_gpu(prob, poison=True)
    assert "ln_pre=pass" in call.plan() and "tile=256x256" in call.plan()
    assert torch.isfinite(got.float()).all()
    rows = sample_rows(4096, 32)
    assert_close(got[rows], oracle_rows(prob, rows), BF16, what="ln_pre full size")
