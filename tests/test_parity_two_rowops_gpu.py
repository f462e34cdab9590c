"""GPU parity of lists with two row reductions (e.g. LayerNorm then softmax: a normalised layer's class
probabilities in one call): the first reduction runs as always, its finalize pass hands fp32 values to a third pass
that reduces again.  Against the oracle, which applies any list in order."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import inputs

from parity import assert_close, oracle_rows, run_gpu

pytestmark = pytest.mark.gpu

F32, BF16, F16, F8 = torch.float32, torch.bfloat16, torch.float16, torch.float8_e4m3fn

LISTS = [
    ["bias", "layernorm", "softmax"],
    ["gelu_tanh", "layernorm", "scale", "logsumexp"],
    ["bias", "layernorm", "relu", "layernorm", "residual"],
    ["softmax", "layernorm"],
    ["scale", "softmax", "scale", "softmax", "bias"],
    ["bias", "residual", "store", "layernorm", "gelu_erf", "softmax"],
]


@pytest.mark.parametrize("kinds", LISTS)
@pytest.mark.parametrize("dtype,variant,split,M,N,K", [
    (BF16, "tiled256", 0, 300, 520, 256), (BF16, "tiled128", 0, 77, 1028, 128), (BF16, "tiled128", 3, 64, 260, 1536),
    (BF16, "general", 0, 45, 77, 50), (BF16, "skinny", 0, 32, 4096, 256), (BF16, "thin", 0, 5, 132, 264), (BF16, "auto", 0, 1, 5000, 512),
    (F32, "auto", 0, 130, 300, 96), (F32, "tiled128", 0, 200, 132, 64), (F16, "auto", 0, 257, 264, 320), (F8, "auto", 0, 300, 516, 512),
])
def test_two_row_reductions_match_oracle(kinds, dtype, variant, split, M, N, K):
    if variant == "thin" and "store" in kinds and N % 4:
        pytest.skip("not a shape of this case")
    prob = inputs.random_problem(61, M, N, K, dtype, kinds)
    print("[case] two row ops", kinds, dtype, variant, split, M, N, K, flush=True)
    got, call = run_gpu(prob, variant, split=split, poison=True)
    assert call.workspace_needed >= M * N * 4
    ref = oracle_rows(prob)
    assert got.shape == ref.shape
    assert_close(got, ref, dtype, call.plan())
    if kinds[-1] == "softmax":
        assert np.abs(got.to(torch.float64).numpy().sum(axis=1) - 1).max() <= (4e-3 if dtype != F32 else 1e-5)


def test_layernorm_then_softmax_at_a_classifier_shape():
    """A vocabulary-sized second reduction (32 rows, 32768 columns) on the skinny kernel's plan."""
    prob = inputs.random_problem(62, 32, 32768, 1024, BF16, ["layernorm", "softmax"])
    got, call = run_gpu(prob, poison=True)
    assert "skinny" in call.plan(), call.plan()
    assert_close(got, oracle_rows(prob), BF16, call.plan())
