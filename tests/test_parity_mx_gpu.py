"""GPU parity of block-scaled fp8 problems (OCP microscaling, MXFP8): x and W in e4m3 with one power-of-two scale per
32 consecutive k, products summed on the matrix instruction's block-scaled form.  The oracle multiplies the values the
stored operands stand for (its decoder is pinned to the format's definition on the CPU side), so the kernel is held to
the ordinary accumulate-and-round tolerance of a bf16 output."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import binding, inputs

from parity import assert_close, oracle_rows, run_gpu, sample_rows

pytestmark = pytest.mark.gpu

F8, BF16 = torch.float8_e4m3fn, torch.bfloat16


def announce(*a):
    print("[case]", *a, flush=True)


@pytest.mark.parametrize("variant,split,M,N,K", [
    ("tiled256", 0, 256, 256, 128), ("tiled256", 0, 300, 520, 384), ("tiled256", 0, 513, 772, 256), ("tiled256", 0, 200, 264, 1024),
    ("tiled128", 0, 128, 128, 256), ("tiled128", 0, 77, 132, 128), ("tiled128", 0, 130, 132, 640), ("tiled128", 0, 64, 128, 1024),
    ("auto", 0, 1, 16, 128), ("auto", 0, 33, 2052, 1024), ("auto", 0, 1030, 260, 512),
    ("tiled256", 3, 300, 260, 1024), ("tiled128", 4, 64, 132, 2048), ("tiled128", 2, 17, 516, 256),
])
def test_block_scaled_integer_inputs_are_bit_exact(variant, split, M, N, K):
    """Small integers times powers of two from 1/4 to 4: every product and every partial sum is exact in fp32, so any
    difference is an indexing error: which scale byte a lane hands to the instruction for which 32 k values, the
    order of the two 16-byte pieces in the upper lane half, the K step a scale dword belongs to, rows past the edge."""
    prob = inputs.random_problem(51, M, N, K, F8, ["bias", "relu", "scale", "residual"], integer=True, mx=True)
    announce("mx integer exact", variant, split, M, N, K)
    got, call = run_gpu(prob, variant, split=split, poison=True)
    assert "_f8mx_" in call.plan(), call.plan()
    ref = torch.from_numpy(oracle_rows(prob)).to(BF16)      # the exact value, rounded once to bf16 as the kernel rounds it
    assert torch.equal(got, ref), call.plan()


@pytest.mark.parametrize("kinds", [
    ["bias", "gelu_erf"], ["scale", "bias", "gelu_tanh", "layernorm"], ["softmax"], ["bias", "residual", "layernorm", "relu"],
    ["scale", "logsumexp"], ["bias", "store", "layernorm"], ["bias", "relu", "scale", "residual"],
])
@pytest.mark.parametrize("M,N,K", [(300, 520, 512), (64, 1028, 2048), (1000, 132, 128)])
def test_block_scaled_chains_match_oracle(kinds, M, N, K):
    """Normal data whose magnitude changes by up to 2^12 from one block of 32 to the next, quantised by the format's
    own recipe: without the scales (or with a neighbour's) the result is off by orders of magnitude."""
    prob = inputs.random_problem(53, M, N, K, F8, kinds, mx=True)
    announce("mx chain", kinds, M, N, K)
    got, call = run_gpu(prob, poison=True)
    assert "_f8mx_" in call.plan()
    assert_close(got, oracle_rows(prob), F8, what="mx %s %s" % (kinds, call.plan()))


def test_block_scaled_full_size_sampled_rows():
    """The benchmark's shape (4096^3 with the bias / relu / scale / residual chain) in the launch configuration the
    benchmark times, rows sampled from every tile row."""
    prob = inputs.random_problem(57, 4096, 4096, 4096, F8, ["bias", "relu", "scale", "residual"], mx=True)
    announce("mx full size")
    got, call = run_gpu(prob, poison=True)
    assert "_f8mx_" in call.plan() and "tile=256x256" in call.plan()
    assert torch.isfinite(got.float()).all()
    rows = sample_rows(4096, 48)
    assert_close(got[rows], oracle_rows(prob, rows), F8, what="mx full size")


def test_scale_tensors_are_checked_by_the_binding():
    prob = inputs.random_problem(59, 64, 128, 256, F8, ["bias"], mx=True)
    dev = "cuda:0"
    x, w, b = prob.x.to(dev), prob.w.to(dev), prob.b.to(dev)
    sx, sw = prob.epilogue[0][1].to(dev), prob.epilogue[0][2].to(dev)
    with pytest.raises(ValueError):
        binding.Call(x, w, b, [("mxscale", sx[:, :4], sw), ("bias",)])
    with pytest.raises(ValueError):
        binding.Call(x, w, b, [("mxscale", sx.to(torch.int8), sw), ("bias",)])
    with pytest.raises(ValueError):
        binding.Call(x, w, b, [("mxscale", sx, sw.cpu()), ("bias",)])
    with pytest.raises(binding.FleError):
        binding.Call(x, w, b, [("bias",), ("mxscale", sx, sw)])
