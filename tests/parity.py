"""Shared helpers of the GPU parity tests: run a Problem through the C-ABI library,
run the same values through the CPU oracle, and compare element by element.

Pass criterion (the allclose form of the paper's Appendix A, with the trusted side on the
right and the absolute part scaled to the output's magnitude):
    |gpu - ref| <= tol * (s + |ref|),   s = min(1, RMS(ref)),
with tol = 1e-4 for fp32 problems, 2e-2 for bf16 problems and 4e-3 for fp16 problems (the same multiple of
the output rounding bound, 2^-11 against bf16's 2^-9, as the bf16 figure).
The attention kernel gets one more term per element, 2 u * sum_j p_j |v_j| with u the rounding unit of the
storage dtype: the kernel rounds the probabilities to the storage dtype for the second product while the
row sum keeps the unrounded ones, two relative errors of at most u on every weight of the convex
combination.  The oracle evaluates that sum itself (attention over |v|), so a late causal row, whose output
averages to a few hundredths of the values' size, is checked against its own size plus this bound.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2511_16964_amd import binding, inputs

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2, torch.float16: 4e-3, torch.float8_e4m3fn: 2e-2}   # (fp8 problems: bf16 out, exact products)


def to_dev(t, dev="cuda:0"):
    return None if t is None else t.to(dev)


def dev_epilogue(ep, dev="cuda:0"):
    return [tuple(to_dev(a, dev) if isinstance(a, torch.Tensor) else a for a in e) for e in ep]


def make_call(prob: inputs.Problem, variant="auto", **kw) -> binding.Call:
    return binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), dev_epilogue(prob.epilogue),
                        variant=variant, **kw)


def run_gpu(prob: inputs.Problem, variant="auto", poison=False, **kw):
    """poison: hand the call an output filled with NaN, so that an element the kernels never wrote shows up
    in the result (a fresh torch.empty may hold anything, including plausible numbers)."""
    if poison:
        lse = bool(prob.epilogue) and prob.epilogue[-1][0] == "logsumexp"
        kw["out"] = torch.full((prob.M,) if lse else (prob.M, prob.N), float("nan"), dtype=inputs.io_dtype(prob.x.dtype), device="cuda:0")
    call = make_call(prob, variant, **kw)
    out = call.run()
    torch.cuda.synchronize()
    return out.cpu(), call


def oracle_rows(prob: inputs.Problem, rows=None) -> np.ndarray:
    """Oracle result for all rows, or for the listed rows only (every op is row-local)."""
    x = prob.x if rows is None else prob.x[rows]
    x64, w64, ep = inputs.to_f64(x), inputs.to_f64(prob.w), prob.epilogue
    if ep and ep[0][0] == "mxscale":   # block-scaled operands: the oracle multiplies the values they stand for
        sx = ep[0][1] if rows is None else ep[0][1][rows]
        x64, w64, ep = oracle.mx_dequantize(x64, sx.numpy()), oracle.mx_dequantize(w64, ep[0][2].numpy()), ep[1:]
    if ep and ep[0][0] == "layernorm_pre":   # LayerNorm of x over K in front of the multiplication
        x64, ep = oracle.layernorm_rows(x64, inputs.to_f64(ep[0][1]), inputs.to_f64(ep[0][2]), ep[0][3]), ep[1:]
    return oracle.fused_linear_epilogue(x64, w64, inputs.to_f64(prob.b), inputs.epilogue_f64(ep, rows))


def excess(got: np.ndarray, ref: np.ndarray, tol: float, s=None, extra=None):
    """(worst violation of the criterion (<= 0 passes), max abs error, RMS-scale s).  extra: a further
    per-element allowance (an array like ref), added to tol * (s + |ref|)."""
    if s is None:
        s = min(1.0, float(np.sqrt(np.mean(ref * ref)))) if ref.size else 1.0
    err = np.abs(got - ref)
    if ref.size == 0:
        return 0.0, 0.0, s
    allow = tol * (s + np.abs(ref))
    if extra is not None:
        allow = allow + extra
    return float(np.max(err - allow)), float(err.max()), s


# The attention block stores two intermediates (qkv and the attention output) in the storage dtype, as the
# eager composition does, before the final rounding: three independent roundings of the same relative size in
# sequence, so its allowance is sqrt(3) times that of a single fused call.
BLOCK_FACTOR = 3.0 ** 0.5


# Rounding unit of the probabilities in the attention kernel (the storage dtype's), times two: see the header.
P_ROUND = {torch.bfloat16: 2.0 ** -8, torch.float16: 2.0 ** -10}


def attention_reference(q, k, v, causal, dtype, scale=None, first_query=0):
    """(oracle result, per-element extra allowance) of attention over float64 q [B,T,H,D] and k, v [B,Tk,H,D]."""
    ref = oracle.attention(q, k, v, causal, scale, first_query=first_query)
    weight = oracle.attention(q, k, np.abs(v), causal, scale, first_query=first_query)   # sum_j p_j |v_j|
    return ref, P_ROUND[dtype] * weight


def assert_close(got_t: torch.Tensor, ref: np.ndarray, dtype, what="", factor=1.0, s=None, extra=None):
    got = got_t.to(torch.float64).numpy()
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite GPU output " + what
    worst, maxerr, s = excess(got, ref, TOL[dtype] * factor, s, extra)
    assert worst <= 0, "%s: criterion exceeded by %.3e (max |err| %.3e, s %.3e)" % (what, worst, maxerr, s)
    return maxerr


def sample_rows(M: int, count: int, tile: int = 256, seed: int = 7):
    """Row sample that holds the first and last row of the matrix and of some tiles, at least one seeded row of
    every tile row (so that no row of tiles goes unchecked), and seeded rows up to `count`."""
    rng = np.random.default_rng(seed)
    rows = {0, M - 1, min(M - 1, tile - 1), min(M - 1, tile), min(M - 1, 31), min(M - 1, 32),
            max(0, M - tile), max(0, M - tile - 1)}
    for lo in range(0, M, tile):
        rows.add(int(rng.integers(lo, min(M, lo + tile))))
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
