"""The pass criteria of the GPU parity tests, exercised on the CPU with planted mistakes (in copies of the
oracle's own results): what the criteria must let through and what they must catch."""
import numpy as np
import torch

import oracle
from paper_2511_16964_amd import inputs

from parity import TOL, attention_reference, excess

BF16 = torch.bfloat16


def late_causal_rows():
    """Attention outputs of the last queries of a causal row of 1024 tokens: averages over ~1000 value rows,
    a few hundredths of the values' size."""
    qkv = inputs.make_qkv(5, 1, 1024, 2, 32, BF16)
    f = inputs.to_f64(qkv)
    ref, extra = attention_reference(f[:, :, 0], f[:, :, 1], f[:, :, 2], True, BF16, first_query=1000)
    return ref, extra


def test_attention_criterion_scales_with_the_row():
    ref, extra = late_causal_rows()
    rms = float(np.sqrt(np.mean(ref * ref)))
    assert rms < 0.06                                   # the premise: late rows are small
    assert float(extra.max()) < 5e-3                    # the rounding term is a fraction of them, not a flat 2e-2
    # rounding to the storage dtype passes
    rounded = torch.from_numpy(ref).to(BF16).to(torch.float64).numpy()
    assert excess(rounded, ref, TOL[BF16], extra=extra)[0] <= 0
    # a halved output row fails, and so does a row replaced by zeros (both passed a flat 2e-2 allowance)
    for factor in (0.5, 0.0):
        bad = ref.copy()
        bad[0, 3] *= factor
        err = np.abs(bad - ref)[0, 3]
        flat_ok = err <= 2e-2 * (1.0 + np.abs(ref[0, 3]))            # a flat allowance of 2e-2 (absolute part 1)
        new_ok = err <= TOL[BF16] * (rms + np.abs(ref[0, 3])) + extra[0, 3]
        assert flat_ok.mean() >= new_ok.mean() + 0.2                 # ... lets far more of the damaged row through
        assert new_ok.mean() < 0.3 and excess(bad, ref, TOL[BF16], extra=extra)[0] > 0
    # a wrong sign on one element of ordinary size fails
    bad = ref.copy()
    i = np.unravel_index(np.argmax(np.abs(ref)), ref.shape)
    bad[i] = -bad[i]
    assert excess(bad, ref, TOL[BF16], extra=extra)[0] > 0


def test_fused_call_criterion_catches_a_zeroed_softmax_row():
    """Softmax outputs of size 1/N: the absolute part of the criterion scales with the output's RMS, so an
    all-zero row does not pass as 'within 2e-2'."""
    rng = np.random.default_rng(0)
    z = rng.standard_normal((4, 4096))
    ref = oracle.fused_linear_epilogue(z, np.eye(4096), None, [("softmax",)])
    rounded = torch.from_numpy(ref).to(BF16).to(torch.float64).numpy()
    assert excess(rounded, ref, TOL[BF16])[0] <= 0
    bad = ref.copy()
    bad[2] = 0.0
    assert np.abs(bad - ref).max() < 2e-2
    assert excess(bad, ref, TOL[BF16])[0] > 0
