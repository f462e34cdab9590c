"""fle_run_static (the entry point for callers that cannot allocate: the library's static scratch array
stands in for the workspace) against fle_run, through the C ABI.  Both plan the same kernels, so the
results must be bit-identical; each case runs two calls in a row on the shared array, the second with a
smaller input, and the larger call is checked against the oracle as well."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2511_16964_amd import binding, inputs

from parity import assert_close, make_call, oracle_rows

pytestmark = pytest.mark.gpu

F32, BF16 = torch.float32, torch.bfloat16

CASES = [
    # (kinds, dtype, variant, split, (M, N, K) of the first call, (M, N, K) of the second)
    (["bias", "gelu_tanh", "layernorm"], BF16, "tiled", 0, (520, 1032, 512), (96, 264, 128)),     # partials in scratch
    (["softmax"], BF16, "skinny", 0, (32, 4096, 1024), (7, 520, 256)),                              # partials; split K slabs when planned
    (["bias", "relu"], BF16, "tiled", 4, (256, 512, 2048), (64, 128, 1024)),                        # fp32 slabs in scratch
    (["scale", "logsumexp"], F32, "general", 0, (77, 333, 50), (5, 31, 17)),                        # partials only
]


@pytest.mark.parametrize("kinds,dtype,variant,split,big,small", CASES)
def test_static_scratch_equals_workspace_call(kinds, dtype, variant, split, big, small):
    for i, (M, N, K) in enumerate((big, small)):
        prob = inputs.random_problem(31 + i, M, N, K, dtype, kinds)
        print("[case] fle_run_static", kinds, dtype, variant, split, M, N, K, flush=True)
        ref_call = make_call(prob, variant, split=split)
        ref = ref_call.run().clone()
        torch.cuda.synchronize()
        assert ref_call.workspace_needed > 0, "test premise: the problem uses scratch"
        call = make_call(prob, variant, split=split, out=torch.full_like(ref, float("nan")),
                         workspace=torch.empty(0, dtype=torch.uint8, device="cuda:0"))
        call._p.workspace, call._p.workspace_bytes = None, 0      # the entry point must not need them
        got = call.run_static()
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), "fle_run_static differs from fle_run"
        if i == 0:
            assert_close(got.cpu(), oracle_rows(prob), dtype, "fle_run_static")


def test_static_scratch_rejects_what_does_not_fit():
    """A problem whose scratch exceeds the array is refused on the host; nothing is enqueued."""
    M, N, K = 4096, 8192, 64      # fp32 staging of [M, N] (a trailing residual that aliases out): 128 MiB
    x = torch.zeros(M, K, dtype=BF16, device="cuda:0")
    w = torch.zeros(N, K, dtype=BF16, device="cuda:0")
    out = torch.zeros(M, N, dtype=BF16, device="cuda:0")
    call = binding.Call(x, w, None, [("layernorm", None, None, 1e-5), ("residual", out)], out=out)
    assert call.workspace_needed > binding.STATIC_SCRATCH_BYTES
    with pytest.raises(binding.FleError) as e:
        call.run_static()
    assert e.value.status == 6 and "static array" in str(e.value)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
