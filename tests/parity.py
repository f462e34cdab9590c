"""Shared helpers of the GPU parity tests: run a Problem through the C-ABI library,
run the same values through the CPU oracle, and compare element by element.

Pass criterion (the allclose form of the paper's Appendix A, with the trusted side on the
right and the absolute part scaled to the output's magnitude):
    |gpu - ref| <= tol * (s + |ref|),   s = min(1, RMS(ref))   (attention kernel alone: s = min(1, RMS(v))),
with tol = 1e-4 for fp32 problems, 2e-2 for bf16 problems and 4e-3 for fp16 problems (the same multiple of
the output rounding bound, 2^-11 against bf16's 2^-9, as the bf16 figure).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2511_16964_amd import binding, inputs

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2, torch.float16: 4e-3}


def to_dev(t, dev="cuda:0"):
    return None if t is None else t.to(dev)


def dev_epilogue(ep, dev="cuda:0"):
    return [tuple(to_dev(a, dev) if isinstance(a, torch.Tensor) else a for a in e) for e in ep]


def make_call(prob: inputs.Problem, variant="auto", **kw) -> binding.Call:
    return binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), dev_epilogue(prob.epilogue),
                        variant=variant, **kw)


def run_gpu(prob: inputs.Problem, variant="auto", **kw):
    call = make_call(prob, variant, **kw)
    out = call.run()
    torch.cuda.synchronize()
    return out.cpu(), call


def oracle_rows(prob: inputs.Problem, rows=None) -> np.ndarray:
    """Oracle result for all rows, or for the listed rows only (every op is row-local)."""
    x = prob.x if rows is None else prob.x[rows]
    return oracle.fused_linear_epilogue(inputs.to_f64(x), inputs.to_f64(prob.w), inputs.to_f64(prob.b),
                                        inputs.epilogue_f64(prob.epilogue, rows))


def excess(got: np.ndarray, ref: np.ndarray, tol: float, s=None):
    """(worst violation of the criterion (<= 0 passes), max abs error, RMS-scale s)."""
    if s is None:
        s = min(1.0, float(np.sqrt(np.mean(ref * ref)))) if ref.size else 1.0
    err = np.abs(got - ref)
    if ref.size == 0:
        return 0.0, 0.0, s
    return float(np.max(err - tol * (s + np.abs(ref)))), float(err.max()), s


# The attention block stores two intermediates (qkv and the attention output) in the storage dtype, as the
# eager composition does, before the final rounding: three independent roundings of the same relative size in
# sequence, so its allowance is sqrt(3) times that of a single fused call.
BLOCK_FACTOR = 3.0 ** 0.5


def value_scale(v: torch.Tensor) -> float:
    """Absolute scale of the attention kernel's criterion: an output row is a convex combination of value rows,
    so rounding the weights (relative 2^-9 in bf16) moves it by that fraction of the values' magnitude, however
    small the row itself is after averaging; s = min(1, RMS(v)) replaces the RMS of the outputs."""
    return min(1.0, float(v.to(torch.float64).pow(2).mean().sqrt()))


def assert_close(got_t: torch.Tensor, ref: np.ndarray, dtype, what="", factor=1.0, s=None):
    got = got_t.to(torch.float64).numpy()
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite GPU output " + what
    worst, maxerr, s = excess(got, ref, TOL[dtype] * factor, s)
    assert worst <= 0, "%s: criterion exceeded by %.3e (max |err| %.3e, s %.3e)" % (what, worst, maxerr, s)
    return maxerr


def sample_rows(M: int, count: int, tile: int = 256, seed: int = 7):
    """Row sample that always holds the first and last row of the matrix and of some tiles."""
    rng = np.random.default_rng(seed)
    rows = {0, M - 1, min(M - 1, tile - 1), min(M - 1, tile), min(M - 1, 31), min(M - 1, 32),
            max(0, M - tile), max(0, M - tile - 1)}
    while len(rows) < min(count, M):
        rows.add(int(rng.integers(0, M)))
    return sorted(rows)


def run_grouped_gpu(gp: inputs.GroupedProblem, variant="auto", offsets=None, shared_out=None, dev="cuda:0"):
    """Run a grouped problem through the C ABI.  ``offsets`` overrides the device array (the library
    never sees the host list)."""
    off = torch.tensor(gp.offsets if offsets is None else offsets, dtype=torch.int64, device=dev)
    call = binding.Call(to_dev(gp.x, dev), to_dev(gp.w, dev), to_dev(gp.b, dev), dev_epilogue(gp.epilogue, dev),
                        out=shared_out, variant=variant, offsets=off)
    out = call.run()
    torch.cuda.synchronize()
    return out.cpu(), call


def oracle_grouped(gp: inputs.GroupedProblem, rows=None) -> np.ndarray:
    """Oracle result of a grouped problem: all rows, or only the listed rows (each row goes through its
    own group's weights as a group of one row)."""
    if rows is None:
        return oracle.grouped_fused_linear_epilogue(inputs.to_f64(gp.x), inputs.to_f64(gp.w), inputs.to_f64(gp.b), gp.offsets,
                                                    inputs.epilogue_f64(gp.epilogue))
    rows = list(rows)
    owner = np.searchsorted(np.asarray(gp.offsets[1:]), np.asarray(rows), side="right")
    out = [None] * len(rows)
    for g in sorted(set(int(o) for o in owner)):      # one oracle call per group that owns sampled rows
        idx = [i for i, o in enumerate(owner) if o == g]
        sel = [rows[i] for i in idx]
        b = None if gp.b is None else (gp.b[g] if gp.b.dim() == 2 else gp.b)
        res = oracle.fused_linear_epilogue(inputs.to_f64(gp.x[sel]), inputs.to_f64(gp.w[g]), inputs.to_f64(b),
                                           inputs.epilogue_f64(gp.epilogue, sel))
        for i, r in zip(idx, res):
            out[i] = r
    return np.stack(out, axis=0)
