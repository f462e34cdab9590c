"""CPU float64 oracle for fused_linear_epilogue -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package.  It imports nothing from the GPU package and shares no
code with it.  The arithmetic lives in ``fle_oracle.c`` (plain C, float64);
this module only compiles it with gcc, loads it with ctypes and marshals
numpy arrays.

The operator is the unfused "gold" composition of the paper's evaluator
(Appendix A, Correctness): matmul, then each listed op with PyTorch-eager
semantics, evaluated in float64 on exactly the input values the GPU receives.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fle_oracle.c")
_LIB = os.path.join(_HERE, "libfle_oracle.so")

# op kinds, in the numbering of fle_oracle.c
BIAS, SCALE, RELU, GELU_ERF, GELU_TANH, RESIDUAL, LAYERNORM, SOFTMAX, LOGSUMEXP, STORE = range(10)
_KINDS = {
    "bias": BIAS, "scale": SCALE, "relu": RELU, "gelu_erf": GELU_ERF, "gelu_tanh": GELU_TANH,
    "residual": RESIDUAL, "layernorm": LAYERNORM, "softmax": SOFTMAX, "logsumexp": LOGSUMEXP, "store": STORE,
}


class _Op(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int32),
        ("alpha", ctypes.c_double),
        ("p0", ctypes.c_void_p),
        ("p1", ctypes.c_void_p),
        ("ld", ctypes.c_int64),
    ]


def build(force: bool = False) -> str:
    """Compile fle_oracle.c into libfle_oracle.so (baseline x86-64, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=gnu11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.fle_oracle_run.restype = ctypes.c_int
        lib.fle_oracle_run.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
            ctypes.POINTER(_Op), ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32]
        lib.fle_oracle_attention.restype = ctypes.c_int
        lib.fle_oracle_attention.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_int32, ctypes.c_double, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32]
        lib.fle_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Threads the oracle's row loop uses by default."""
    return int(_load().fle_oracle_threads())


def _f64(a):
    if a is None:
        return None
    a = np.asarray(a)
    if a.dtype != np.float64:
        raise TypeError("the oracle takes float64 arrays only (upcast the rounded inputs exactly)")
    return np.ascontiguousarray(a)


def fused_linear_epilogue(x, w, b, epilogue, n_threads: int = 0) -> np.ndarray:
    """float64 gold result of ``epilogue(x @ w.T)``.

    x [M,K], w [N,K], b [N] or None: float64 numpy arrays (already holding the
    fp32- or bf16-rounded values the GPU gets; the upcast is exact).
    epilogue: ordered list of tuples
        ("bias",) ("scale", alpha) ("relu",) ("gelu_erf",) ("gelu_tanh",)
        ("residual", r[M,N]) ("layernorm", gamma|None, beta|None, eps)
        ("softmax",) ("logsumexp",)       -- logsumexp only as the last entry.
        ("store", t[M,N])                 -- t (a float64 array, written in place) receives a copy of the
                                             values as they stand at this point of the chain; the chain
                                             goes on unchanged.  This is how a producer hands over both a
                                             value and its normalisation (x + f(x) and LayerNorm of it).
    alpha and eps cross the GPU boundary as fp32, so they are rounded to fp32
    here too (Appendix A compares like with like).
    Returns [M,N] float64, or [M] when the list ends in logsumexp.
    """
    x, w, b = _f64(x), _f64(w), _f64(b)
    if x.ndim != 2 or w.ndim != 2 or x.shape[1] != w.shape[1]:
        raise ValueError("x must be [M,K] and w [N,K]")
    M, K = x.shape
    N = w.shape[0]
    keep = [x, w, b]
    ops = (_Op * max(1, len(epilogue)))()
    for i, e in enumerate(epilogue):
        kind = _KINDS[e[0]]
        ops[i].kind = kind
        if kind == SCALE:
            ops[i].alpha = float(np.float32(e[1]))
        elif kind == RESIDUAL:
            r = _f64(e[1])
            if r.shape != (M, N):
                raise ValueError("residual must be [M,N]")
            keep.append(r)
            ops[i].p0 = r.ctypes.data
            ops[i].ld = N
        elif kind == STORE:
            t = e[1]
            if not isinstance(t, np.ndarray) or t.dtype != np.float64 or t.shape != (M, N) or not t.flags.c_contiguous:
                raise ValueError("store needs a C-contiguous float64 array [M,N]")
            keep.append(t)
            ops[i].p0 = t.ctypes.data
            ops[i].ld = N
        elif kind == LAYERNORM:
            g, be = _f64(e[1]), _f64(e[2])
            keep += [g, be]
            ops[i].p0 = g.ctypes.data if g is not None else None
            ops[i].p1 = be.ctypes.data if be is not None else None
            ops[i].alpha = float(np.float32(e[3]))
    lse = bool(epilogue) and epilogue[-1][0] == "logsumexp"
    out = np.empty((M,) if lse else (M, N), dtype=np.float64)
    rc = _load().fle_oracle_run(
        M, N, K, x.ctypes.data, K, w.ctypes.data, K, b.ctypes.data if b is not None else None,
        ops, len(epilogue), out.ctypes.data, N, int(n_threads))
    if rc != 0:
        raise ValueError("fle_oracle_run rejected the arguments (code %d)" % rc)
    return out


def layernorm_rows(x, gamma=None, beta=None, eps: float = 1e-5) -> np.ndarray:
    """LayerNorm over the last axis of x [M, K], the definition written out in float64 (PyTorch-eager semantics:
    biased variance, eps inside the square root): (x - mean) / sqrt(var + eps) * gamma + beta.  This is what a
    LayerNorm in front of the linear layer hands to the multiplication."""
    x = _f64(x)
    eps = float(np.float32(eps))   # (eps crosses the GPU boundary as fp32, as for the row op)
    mean = x.mean(axis=1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=1, keepdims=True)
    y = (x - mean) / np.sqrt(var + eps)
    if gamma is not None:
        y = y * _f64(gamma)[None, :]
    if beta is not None:
        y = y + _f64(beta)[None, :]
    return y


def mx_dequantize(elems, scales) -> np.ndarray:
    """The values a block-scaled operand stands for (OCP Microscaling Formats specification, MXFP8): elems [R, K]
    are the stored elements (already upcast exactly), scales [R, K/32] one byte per block of 32 consecutive
    elements of a row, E8M0: the block's values are multiplied by 2^(byte - 127); byte 255 makes them NaN.
    The product is exact in float64 (an 8-bit element times a power of two within double's exponent range)."""
    elems = _f64(elems)
    sc = np.asarray(scales)
    if sc.dtype != np.uint8 or elems.ndim != 2 or sc.shape != (elems.shape[0], elems.shape[1] // 32) or elems.shape[1] % 32:
        raise ValueError("need elems [R, K], K a multiple of 32, and uint8 scales [R, K/32]")
    factor = np.ldexp(1.0, sc.astype(np.int64) - 127)
    factor[sc == 255] = np.nan
    return elems * np.repeat(factor, 32, axis=1)


def grouped_fused_linear_epilogue(x, w, b, offsets, epilogue, n_threads: int = 0) -> np.ndarray:
    """float64 gold result of the grouped form: the loop over groups written out.

    Rows ``offsets[g] .. offsets[g+1]-1`` of x go through ``fused_linear_epilogue`` with
    ``w[g]`` (and ``b[g]``), exactly the per-expert loop that the paper's appendix on outlier
    tasks (Level 5, the mixture-of-experts task) says the optimised solutions replace by one
    grouped matrix multiplication; the grouping never changes a row's result.

    x [M,K]; w [G,N,K]; b [G,N], [N] (shared) or None; offsets: G+1 non-decreasing integers
    from 0 to M; residual operands in the epilogue are [M,N].  Returns [M,N], or [M] when the
    list ends in logsumexp.
    """
    x, w = _f64(x), _f64(w)
    b = _f64(b)
    if x.ndim != 2 or w.ndim != 3 or x.shape[1] != w.shape[2]:
        raise ValueError("x must be [M,K] and w [G,N,K]")
    offsets = [int(o) for o in offsets]
    G, N = w.shape[0], w.shape[1]
    M = x.shape[0]
    if len(offsets) != G + 1 or offsets[0] != 0 or offsets[-1] != M or any(a > c for a, c in zip(offsets, offsets[1:])):
        raise ValueError("offsets must be G+1 non-decreasing integers from 0 to M")
    lse = bool(epilogue) and epilogue[-1][0] == "logsumexp"
    out = np.empty((M,) if lse else (M, N), dtype=np.float64)
    for g in range(G):
        lo, hi = offsets[g], offsets[g + 1]
        if hi == lo:
            continue
        # [M,N] operands are cut to the group's rows (a store target as a view, written in place)
        ep = [(e[0], np.asarray(e[1])[lo:hi]) if e[0] in ("residual", "store") else e for e in epilogue]
        bg = None if b is None else (b[g] if b.ndim == 2 else b)
        out[lo:hi] = fused_linear_epilogue(x[lo:hi], w[g], bg, ep, n_threads)
    return out


def attention(q, k, v, causal, scale=None, n_threads: int = 0, first_query: int = 0) -> np.ndarray:
    """float64 gold result of scaled dot-product attention, token-major.

    q: [B, T, H, D], k and v: [B, Tk, H, D] float64 (views are accepted, e.g. the three thirds of a
    fused QKV projection's output).  With Tk != T and a causal mask the queries are the last T of
    the Tk positions (query t stands at position t + Tk - T; needs Tk >= T). scale defaults to
    1/sqrt(D) and is rounded to fp32 as it is when it crosses the GPU boundary.  causal: False / 0:
    every key; True / 1: query t sees keys 0..t only; G > 1: the same over groups of G consecutive
    tokens, query t sees keys 0 .. (t // G + 1) * G - 1 (the mask the paper's attention solutions
    apply on the fly, appendix on Level 5 outliers).  Returns [B, T, H, D]; with first_query = t0 only queries t0 .. T-1 are
    evaluated (against all their keys) and [B, T - t0, H, D] is returned.
    """
    q, k, v = (np.asarray(a) for a in (q, k, v))
    if q.ndim != 4 or k.ndim != 4 or k.shape != v.shape or q.shape[0] != k.shape[0] or q.shape[2:] != k.shape[2:]:
        raise ValueError("q must be [B,T,H,D] and k, v [B,Tk,H,D]")
    for a in (q, k, v):
        if a.dtype != np.float64:
            raise TypeError("the oracle takes float64 arrays only")
    B, T, H, D = q.shape
    Tk = k.shape[1]
    q2 = np.ascontiguousarray(q).reshape(B * T, H * D)
    k2, v2 = (np.ascontiguousarray(a).reshape(B * Tk, H * D) for a in (k, v))
    sc = float(np.float32(1.0 / np.sqrt(D) if scale is None else scale))
    out = np.full((B * T, H * D), np.nan, dtype=np.float64)
    rc = _load().fle_oracle_attention(
        B, H, T, Tk, D, q2.ctypes.data, H * D, k2.ctypes.data, H * D, v2.ctypes.data, H * D,
        int(causal), sc, out.ctypes.data, H * D, int(first_query), int(n_threads))
    if rc != 0:
        raise ValueError("fle_oracle_attention rejected the arguments (code %d)" % rc)
    return out.reshape(B, T, H, D)[:, int(first_query):]


def attention_block(x, w_qkv, b_qkv, w_o, b_o, heads: int, causal, residual=None, n_threads: int = 0) -> np.ndarray:
    """float64 gold result of a self-attention block: the unfused composition.

    qkv = x w_qkv^T + b_qkv is cut into thirds q | k | v along its columns, each third into
    `heads` heads of D = C / heads columns; attention runs per head; the heads' outputs, side by
    side again, go through the output projection w_o (+ b_o, + residual).  This is the block whose
    fusion (projections included) the paper's task-wise analysis reports as its largest recurring
    speedup.  x [B,T,C]; w_qkv [3C,C]; b_qkv [3C] or None; w_o [C,C]; b_o [C] or None;
    residual [B,T,C] or None.  Returns [B,T,C].
    """
    x = _f64(x)
    B, T, C = x.shape
    if C % heads:
        raise ValueError("C must be a multiple of heads")
    D = C // heads
    qkv = fused_linear_epilogue(x.reshape(B * T, C), w_qkv, b_qkv, [("bias",)] if b_qkv is not None else [], n_threads)
    qkv = qkv.reshape(B, T, 3, heads, D)
    o = attention(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], causal, None, n_threads)
    ep = ([("bias",)] if b_o is not None else []) + ([("residual", _f64(residual).reshape(B * T, C))] if residual is not None else [])
    y = fused_linear_epilogue(o.reshape(B * T, C), w_o, b_o, ep, n_threads)
    return y.reshape(B, T, C)


def transformer_layer(x, n, w_qkv, b_qkv, w_o, b_o, heads: int, causal, ln_mid, w1, b1, w2, b2, ln_out, n_threads: int = 0):
    """float64 gold result of one pre-norm transformer layer, from its normalised input on: the unfused composition.

    The paper's Level-3 style tasks are whole architectures made of such layers (attention block, then a
    perceptron block, each added to the residual stream, each fed by a LayerNorm of it).  With x the residual
    stream [B,T,C] and n [B,T,C] its normalised form (what the previous layer hands over):
        h  = x + attention_block(n)                      (projections, attention, output projection + bias)
        m  = LayerNorm_mid(h)
        x' = h + gelu_erf(m w1^T + b1) w2^T + b2
        n' = LayerNorm_out(x')                           (the next layer's normalised input)
    ln_mid and ln_out are (gamma, beta, eps).  Returns (x', n'), both [B,T,C].
    """
    x = _f64(x)
    B, T, C = x.shape
    h = attention_block(n, w_qkv, b_qkv, w_o, b_o, heads, causal, residual=x, n_threads=n_threads).reshape(B * T, C)
    eye = np.eye(C, dtype=np.float64)   # a LayerNorm alone, written as the epilogue of a product with the identity
    m = fused_linear_epilogue(h, eye, None, [("layernorm", ln_mid[0], ln_mid[1], ln_mid[2])], n_threads)
    u = fused_linear_epilogue(m, w1, b1, [("bias",), ("gelu_erf",)], n_threads)
    x2 = fused_linear_epilogue(u, w2, b2, [("bias",), ("residual", h)], n_threads)
    n2 = fused_linear_epilogue(x2, eye, None, [("layernorm", ln_out[0], ln_out[1], ln_out[2])], n_threads)
    return x2.reshape(B, T, C), n2.reshape(B, T, C)
