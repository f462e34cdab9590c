"""Seeded synthetic inputs for the benchmark configurations.

This module holds no arithmetic of the operator itself: it only draws random
tensors of the stated shapes and distributions and rounds them to the storage
dtype.  Both the GPU tests and the CPU oracle consume exactly these values
(the oracle after an exact upcast to float64).

Generator: ``numpy.random.default_rng(seed)``; draw order per problem is
x, W, b, r, gamma, beta (for the two-call MLP block: x, W1, b1, W2, b2, gamma,
beta).  N(0,1) is ``standard_normal``; U(+-a) is ``uniform(-a, a)``;
N(mu, s) has standard deviation s.  bf16 storage is round-to-nearest-even of
the fp32 draw.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch


@dataclass
class Problem:
    """One call of fused_linear_epilogue: CPU tensors in the storage dtype."""
    name: str
    dtype: torch.dtype
    x: torch.Tensor                 # [M, K]
    w: torch.Tensor                 # [N, K]
    b: torch.Tensor | None          # [N]
    epilogue: list = field(default_factory=list)  # tuples; tensors inside are CPU tensors

    @property
    def M(self): return self.x.shape[0]

    @property
    def N(self): return self.w.shape[0]

    @property
    def K(self): return self.x.shape[1]

    @property
    def flops(self): return 2 * self.M * self.N * self.K


def _normal(rng, shape, mean=0.0, std=1.0):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return a


def _uniform(rng, shape, a):
    return rng.uniform(-a, a, size=shape).astype(np.float32)


def _store(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    return torch.from_numpy(a).to(dtype)


F8 = torch.float8_e4m3fn


def io_dtype(dtype: torch.dtype) -> torch.dtype:
    """Dtype of b, residual / store operands, gamma, beta and out of a problem whose x and W have ``dtype``
    (fp8 problems keep everything but x and W in bf16)."""
    return torch.bfloat16 if dtype == F8 else dtype


# name -> (dtype, M, N, K)
SHAPES = {
    "c1": (torch.float32, 64, 256, 256),
    "c2": (torch.bfloat16, 4096, 4096, 4096),
    "c3": (torch.bfloat16, 8192, 4096, 4096),
    "c4": (torch.bfloat16, 32, 32768, 8192),
    "c5a": (torch.bfloat16, 16384, 16384, 4096),
    "c5b": (torch.bfloat16, 16384, 4096, 16384),
    "f2": (torch.float8_e4m3fn, 4096, 4096, 4096),   # c2 with x and W stored in fp8 (one scale per tensor)
    "p1": (torch.bfloat16, 1, 4096, 4096),            # one token: LayerNorm over K, then Linear + bias + GELU-erf (launch-bound)
    "p2": (torch.bfloat16, 4096, 4096, 4096),         # 4096 tokens: the same normalisation -> projection pair (compute-bound)
    "f3": (torch.float8_e4m3fn, 4096, 4096, 4096),   # ... in block-scaled fp8 (MXFP8: one power-of-two scale per 32 k)
}


def make(name: str, seed: int = 0, M: int | None = None, N: int | None = None,
         K: int | None = None) -> Problem:
    """Build configuration ``name`` ("c1".."c4", "f2"); M, N, K override the shape
    (same distributions, for reduced-size parity cases)."""
    dtype, M0, N0, K0 = SHAPES[name]
    M, N, K = M or M0, N or N0, K or K0
    rng = np.random.default_rng(seed)
    if name == "c1":    # Linear + bias + GELU-erf, fp32
        x = _normal(rng, (M, K)); w = _uniform(rng, (N, K), 1 / 16); b = _uniform(rng, (N,), 1 / 16)
        return Problem(name, dtype, _store(x, dtype), _store(w, dtype), _store(b, dtype),
                       [("bias",), ("gelu_erf",)])
    if name == "c2":    # Linear + bias + ReLU + scale(0.5) + residual, bf16
        x = _normal(rng, (M, K)); w = _uniform(rng, (N, K), 1 / 64); b = _uniform(rng, (N,), 1 / 64)
        r = _normal(rng, (M, N))
        return Problem(name, dtype, _store(x, dtype), _store(w, dtype), _store(b, dtype),
                       [("bias",), ("relu",), ("scale", 0.5), ("residual", _store(r, dtype))])
    if name == "f2":    # c2's layer with fp8 storage: x / sx and W / sw in e4m3 (the largest magnitude maps to 448), scale sx sw first
        x = _normal(rng, (M, K)); w = _uniform(rng, (N, K), 1 / 64); b = _uniform(rng, (N,), 1 / 64)
        r = _normal(rng, (M, N))
        sx, sw = float(np.abs(x).max()) / 448.0, float(np.abs(w).max()) / 448.0
        return Problem(name, dtype, _store(x / np.float32(sx), dtype), _store(w / np.float32(sw), dtype), _store(b, torch.bfloat16),
                       [("scale", float(np.float32(sx * sw))), ("bias",), ("relu",), ("scale", 0.5), ("residual", _store(r, torch.bfloat16))])
    if name in ("p1", "p2"):   # a transformer block's normalisation -> projection pair: LayerNorm(x) W^T + b, GELU-erf
        x = _normal(rng, (M, K), 0.25, 1.0); w = _uniform(rng, (N, K), 1 / 64); b = _uniform(rng, (N,), 1 / 64)
        g = _normal(rng, (K,), 1.0, 0.02); be = _normal(rng, (K,), 0.0, 0.02)
        return Problem(name, dtype, _store(x, dtype), _store(w, dtype), _store(b, dtype),
                       [("layernorm_pre", _store(g, dtype), _store(be, dtype), 1e-5), ("bias",), ("gelu_erf",)])
    if name == "f3":    # c2's layer with block-scaled fp8 storage (the same values as c2 and f2, quantised block by block)
        x = _normal(rng, (M, K)); w = _uniform(rng, (N, K), 1 / 64); b = _uniform(rng, (N,), 1 / 64)
        r = _normal(rng, (M, N))
        (xq, sx), (wq, sw) = mx_quantize(x), mx_quantize(w)
        return Problem(name, dtype, xq, wq, _store(b, torch.bfloat16),
                       [("mxscale", sx, sw), ("bias",), ("relu",), ("scale", 0.5), ("residual", _store(r, torch.bfloat16))])
    if name == "c3":    # Linear + bias + GELU-tanh + LayerNorm, bf16
        x = _normal(rng, (M, K)); w = _uniform(rng, (N, K), 1 / 64); b = _uniform(rng, (N,), 1 / 64)
        g = _normal(rng, (N,), 1.0, 0.02); be = _normal(rng, (N,), 0.0, 0.02)
        return Problem(name, dtype, _store(x, dtype), _store(w, dtype), _store(b, dtype),
                       [("bias",), ("gelu_tanh",),
                        ("layernorm", _store(g, dtype), _store(be, dtype), 1e-5)])
    if name == "c4":    # skinny Linear + row softmax, bf16, no bias
        x = _normal(rng, (M, K)); w = _uniform(rng, (N, K), 1 / math.sqrt(K))
        return Problem(name, dtype, _store(x, dtype), _store(w, dtype), None, [("softmax",)])
    raise KeyError(name)


@dataclass
class MlpBlock:
    """Transformer MLP block as two calls: h = gelu_erf(x W1^T + b1);
    out = layernorm(h W2^T + b2 + x)."""
    x: torch.Tensor      # [T, D]
    w1: torch.Tensor     # [F, D]
    b1: torch.Tensor     # [F]
    w2: torch.Tensor     # [D, F]
    b2: torch.Tensor     # [D]
    gamma: torch.Tensor  # [D]
    beta: torch.Tensor   # [D]
    eps: float = 1e-5

    def call1(self, x=None) -> Problem:
        x = self.x if x is None else x
        return Problem("c5a", x.dtype, x, self.w1, self.b1, [("bias",), ("gelu_erf",)])

    def call2(self, h, x=None) -> Problem:
        x = self.x if x is None else x
        return Problem("c5b", h.dtype, h, self.w2, self.b2,
                       [("bias",), ("residual", x), ("layernorm", self.gamma, self.beta, self.eps)])


def make_mlp(seed: int = 0, T: int = 16384, D: int = 4096, F: int = 16384,
             dtype: torch.dtype = torch.bfloat16) -> MlpBlock:
    rng = np.random.default_rng(seed)
    x = _normal(rng, (T, D))
    w1 = _uniform(rng, (F, D), 1 / math.sqrt(D)); b1 = _uniform(rng, (F,), 1 / math.sqrt(D))
    w2 = _uniform(rng, (D, F), 1 / math.sqrt(F)); b2 = _uniform(rng, (D,), 1 / math.sqrt(F))
    g = _normal(rng, (D,), 1.0, 0.02); be = _normal(rng, (D,), 0.0, 0.02)
    s = lambda a: _store(a, dtype)
    return MlpBlock(s(x), s(w1), s(b1), s(w2), s(b2), s(g), s(be))


def mx_quantize(a: np.ndarray):
    """Stores a float matrix [R, K] (K a multiple of 32) in the OCP microscaling format with e4m3 elements (MXFP8):
    every block of 32 consecutive values of a row gets the power of two 2^e with e = floor(log2(max |v|)) - 8 (8 is
    the exponent of e4m3's largest value, 448 = 1.75 * 2^8; a block of zeros gets the smallest scale), stored as
    the byte e + 127, and its values divided by that scale are rounded to e4m3, saturating at +-448.
    Returns (elements as a float8_e4m3fn tensor [R, K], scales as a uint8 tensor [R, K/32])."""
    R, K = a.shape
    blocks = a.astype(np.float64).reshape(R, K // 32, 32)
    amax = np.abs(blocks).max(axis=2)
    e = np.where(amax > 0, np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - 8, -127).clip(-127, 127).astype(np.int64)
    elems = np.clip(blocks / np.ldexp(1.0, e)[:, :, None], -448.0, 448.0).reshape(R, K)
    return torch.from_numpy(elems.astype(np.float32)).to(F8), torch.from_numpy((e + 127).astype(np.uint8))


def random_problem(seed: int, M: int, N: int, K: int, dtype: torch.dtype, kinds: list[str],
                   integer: bool = False, mx: bool = False, ln_pre: bool = False, x_mean: float = 0.5) -> Problem:
    """A problem with an arbitrary epilogue list, for parity sweeps.  With
    ``integer`` every tensor holds small integers (exactly representable in
    bf16), which makes the elementwise chain bias/relu/scale(0.5)/residual exact.
    ``ln_pre``: the list starts with ("layernorm_pre", gamma[K], beta[K], 1e-5), a LayerNorm of x over K in front of the
    multiplication; the rows of x then have mean ``x_mean`` (and unit deviation), gamma ~ N(1, 0.1), beta ~ N(0, 0.1).
    ``mx`` (fp8 problems, K a multiple of 128): x and W are block-scaled; their magnitudes then vary from one
    block of 32 to the next by up to 2^12 (integer: the scales are random powers of two from 1/4 to 4 and the
    elements small integers, so every product and partial sum is still exact in fp32); the list starts with the
    ("mxscale", scales of x, scales of W) entry."""
    rng = np.random.default_rng(seed)
    if integer:
        ri = lambda shape, a: rng.integers(-a, a + 1, size=shape).astype(np.float32)
        x, w, b = ri((M, K), 2), ri((N, K), 2), ri((N,), 8)
    else:
        x = _normal(rng, (M, K)); w = _uniform(rng, (N, K), 1 / math.sqrt(max(K, 1)))
        b = _uniform(rng, (N,), 0.5)
    ep = []
    io = io_dtype(dtype)
    if ln_pre:
        x = x + np.float32(x_mean)
        ep.append(("layernorm_pre", _store(_normal(rng, (K,), 1.0, 0.1), io), _store(_normal(rng, (K,), 0.0, 0.1), io), 1e-5))
    if mx:
        assert dtype == F8 and K % 128 == 0
        if integer:
            sx = rng.integers(125, 130, size=(M, K // 32)).astype(np.uint8); sw = rng.integers(125, 130, size=(N, K // 32)).astype(np.uint8)
            xq, wq = _store(x, F8), _store(w, F8)
            sx, sw = torch.from_numpy(sx), torch.from_numpy(sw)
        else:
            x = x * np.ldexp(1.0, rng.integers(-6, 7, size=(M, K // 32))).repeat(32, axis=1).astype(np.float32)
            w = w * np.ldexp(1.0, rng.integers(-6, 7, size=(N, K // 32))).repeat(32, axis=1).astype(np.float32)
            (xq, sx), (wq, sw) = mx_quantize(x), mx_quantize(w)
        ep.append(("mxscale", sx, sw))
    for kd in kinds:
        if kd == "scale":
            ep.append(("scale", 0.5 if integer else float(np.float32(rng.uniform(0.25, 2.0)))))
        elif kd == "residual":
            r = ri((M, N), 8) if integer else _normal(rng, (M, N))
            ep.append(("residual", _store(r, io)))
        elif kd == "layernorm":
            g = _normal(rng, (N,), 1.0, 0.1); be = _normal(rng, (N,), 0.0, 0.1)
            ep.append(("layernorm", _store(g, io), _store(be, io), 1e-5))
        elif kd == "store":   # the target: an output, pre-filled so that an unwritten element shows
            ep.append(("store", torch.full((M, N), -7.0, dtype=io)))
        else:
            ep.append((kd,))
    if mx:
        return Problem("random", dtype, xq, wq, _store(b, io), ep)
    return Problem("random", dtype, _store(x, dtype), _store(w, dtype), _store(b, io), ep)


@dataclass
class GroupedProblem:
    """One grouped call: rows offsets[g] .. offsets[g+1]-1 of x belong to group g."""
    dtype: torch.dtype
    x: torch.Tensor                 # [M, K]
    w: torch.Tensor                 # [G, N, K]
    b: torch.Tensor | None          # [G, N]
    offsets: list                   # G + 1 integers, 0 .. M
    epilogue: list = field(default_factory=list)  # residual operands are [M, N]

    @property
    def M(self): return self.x.shape[0]

    @property
    def N(self): return self.w.shape[1]

    @property
    def K(self): return self.x.shape[1]

    @property
    def flops(self): return 2 * self.M * self.N * self.K


def routed_counts(seed: int, M: int, G: int, skew: float = 1.0) -> list[int]:
    """Rows per group for M rows routed to G groups: a multinomial draw whose probabilities come
    from a Dirichlet(skew) draw, the load imbalance of a learned router (small skew: a few hot
    groups and some empty ones; large skew: nearly even)."""
    rng = np.random.default_rng(seed)
    prob = rng.dirichlet(np.full(G, float(skew)))
    return [int(c) for c in rng.multinomial(M, prob)]


def offsets_of(counts) -> list[int]:
    off = [0]
    for c in counts:
        off.append(off[-1] + int(c))
    return off


def random_grouped(seed: int, counts, N: int, K: int, dtype: torch.dtype, kinds: list[str],
                   integer: bool = False, shared_bias: bool = False) -> GroupedProblem:
    """A grouped problem with ``counts[g]`` rows in group g; same value recipes as
    ``random_problem`` (draw order x, W, b, then the epilogue operands)."""
    rng = np.random.default_rng(seed)
    G, M = len(counts), int(sum(counts))
    bshape = (N,) if shared_bias else (G, N)
    if integer:
        ri = lambda shape, a: rng.integers(-a, a + 1, size=shape).astype(np.float32)
        x, w, b = ri((M, K), 2), ri((G, N, K), 2), ri(bshape, 8)
    else:
        x = _normal(rng, (M, K)); w = _uniform(rng, (G, N, K), 1 / math.sqrt(max(K, 1)))
        b = _uniform(rng, bshape, 0.5)
    ep = []
    for kd in kinds:
        if kd == "scale":
            ep.append(("scale", 0.5 if integer else float(np.float32(rng.uniform(0.25, 2.0)))))
        elif kd == "residual":
            r = ri((M, N), 8) if integer else _normal(rng, (M, N))
            ep.append(("residual", _store(r, io_dtype(dtype))))
        elif kd == "layernorm":
            g = _normal(rng, (N,), 1.0, 0.1); be = _normal(rng, (N,), 0.0, 0.1)
            ep.append(("layernorm", _store(g, io_dtype(dtype)), _store(be, io_dtype(dtype)), 1e-5))
        elif kd == "store":   # the target: an output, pre-filled so that an unwritten element shows
            ep.append(("store", torch.full((M, N), -7.0, dtype=io_dtype(dtype))))
        else:
            ep.append((kd,))
    return GroupedProblem(dtype, _store(x, dtype), _store(w, dtype), _store(b, io_dtype(dtype)), offsets_of(counts), ep)


# name -> (dtype, rows M, groups G, N, K, Dirichlet skew of the routing)
GROUPED_SHAPES = {
    "g1": (torch.bfloat16, 32768, 32, 4096, 4096, 1.0),   # a routed training / prefill batch: about 1024 rows per group
    "g2": (torch.bfloat16, 512, 32, 4096, 4096, 1.0),     # a small decoding batch: about 16 rows per group, weight-bound
}


def make_grouped(name: str, seed: int = 0, M: int | None = None, G: int | None = None,
                 N: int | None = None, K: int | None = None) -> GroupedProblem:
    """Grouped benchmark configuration ``name``: Linear + bias + GELU-tanh per group, rows routed by
    ``routed_counts``; M, G, N, K override the shape for reduced-size parity cases."""
    dtype, M0, G0, N0, K0, skew = GROUPED_SHAPES[name]
    M, G, N, K = M or M0, G or G0, N or N0, K or K0
    return random_grouped(seed, routed_counts(seed + 1000, M, G, skew), N, K, dtype, ["bias", "gelu_tanh"])


@dataclass
class MlpChain:
    """A multi-layer perceptron at a tiny batch: layer i is h_i = relu(h_{i-1} W_i^T + b_i), h_0 = x."""
    x: torch.Tensor        # [B, width]
    ws: list               # L tensors [width, width]
    bs: list               # L tensors [width]

    def layer(self, i: int, h: torch.Tensor) -> Problem:
        return Problem("m1.%d" % i, h.dtype, h, self.ws[i], self.bs[i], [("bias",), ("relu",)])


def make_chain(seed: int = 0, batch: int = 1, width: int = 4096, layers: int = 8,
               dtype: torch.dtype = torch.float32) -> MlpChain:
    """Workload m1: x ~ N(0,1); W_i ~ U(+-sqrt(6/width)) (keeps the activations' scale through the
    ReLUs), b_i ~ U(+-0.1); draw order x, then W_i, b_i layer by layer."""
    rng = np.random.default_rng(seed)
    x = _normal(rng, (batch, width))
    ws, bs = [], []
    for _ in range(layers):
        ws.append(_store(_uniform(rng, (width, width), math.sqrt(6.0 / width)), dtype))
        bs.append(_store(_uniform(rng, (width,), 0.1), dtype))
    return MlpChain(_store(x, dtype), ws, bs)


@dataclass
class AttentionProblem:
    """One self-attention block: CPU tensors in the storage dtype."""
    name: str
    dtype: torch.dtype
    heads: int
    causal: bool
    x: torch.Tensor                 # [B, T, C]
    w_qkv: torch.Tensor             # [3C, C], output columns q | k | v
    b_qkv: torch.Tensor | None      # [3C]
    w_o: torch.Tensor               # [C, C]
    b_o: torch.Tensor | None        # [C]
    residual: torch.Tensor | None   # [B, T, C]

    @property
    def flops(self) -> float:
        """Both projections, and the two products of the attention itself over the keys the mask allows."""
        B, T, C = self.x.shape
        pairs = T * (T + 1) / 2 if self.causal else T * T
        return 2.0 * B * T * C * 3 * C + 4.0 * B * pairs * C + 2.0 * B * T * C * C


# name: (dtype, B, T, C, heads, causal) -- a1: a GPT-style causal block, 16 sequences of 2048 tokens
ATTENTION_SHAPES = {
    "a1": (torch.bfloat16, 16, 2048, 2048, 16, True),
}


def make_attention(name: str = "a1", seed: int = 0, B: int | None = None, T: int | None = None, C: int | None = None,
                   heads: int | None = None, causal: bool | None = None, dtype: torch.dtype | None = None,
                   bias: bool = True, residual: bool = True) -> AttentionProblem:
    """x ~ N(0,1); W_qkv ~ N(0, 1/sqrt(C)) so that q, k, v are ~N(0,1) and the scores ~N(0,1) after the
    1/sqrt(D) scale; b_qkv ~ U(+-0.1); W_o ~ N(0, 1/sqrt(C)); b_o ~ U(+-0.1); the residual is x itself
    (the block's input, as in a pre-norm transformer).  Draw order x, W_qkv, b_qkv, W_o, b_o."""
    dt0, B0, T0, C0, H0, c0 = ATTENTION_SHAPES[name]
    dtype = dt0 if dtype is None else dtype
    B, T, C = (B0 if B is None else B), (T0 if T is None else T), (C0 if C is None else C)
    heads = H0 if heads is None else heads
    causal = c0 if causal is None else causal
    rng = np.random.default_rng(seed)
    x = _store(_normal(rng, (B, T, C)), dtype)
    w_qkv = _store(_normal(rng, (3 * C, C), 0.0, 1.0 / math.sqrt(C)), dtype)
    b_qkv = _store(_uniform(rng, (3 * C,), 0.1), dtype)
    w_o = _store(_normal(rng, (C, C), 0.0, 1.0 / math.sqrt(C)), dtype)
    b_o = _store(_uniform(rng, (C,), 0.1), dtype)
    return AttentionProblem(name, dtype, heads, causal, x, w_qkv, b_qkv if bias else None, w_o, b_o if bias else None,
                            x if residual else None)


@dataclass
class LayerProblem:
    """One pre-norm transformer layer from its normalised input on: the attention block of ``attn`` applied
    to n and added to x, LayerNorm (g_mid, be_mid), the perceptron block (w1, b1, GELU-erf, w2, b2) added to
    that, LayerNorm (g_out, be_out) for the next layer."""
    attn: AttentionProblem      # x = the residual stream [B,T,C]; its weights are the block's
    n: torch.Tensor             # [B,T,C]: the normalised stream the previous layer hands over
    g_mid: torch.Tensor
    be_mid: torch.Tensor
    w1: torch.Tensor            # [F,C]
    b1: torch.Tensor
    w2: torch.Tensor            # [C,F]
    b2: torch.Tensor
    g_out: torch.Tensor
    be_out: torch.Tensor
    eps: float = 1e-5

    @property
    def flops(self) -> float:
        B, T, C = self.n.shape
        return self.attn.flops + 4.0 * B * T * C * self.w1.shape[0]


def make_layer(name: str = "a1", seed: int = 0, F: int | None = None, **kw) -> LayerProblem:
    """The attention block of ``make_attention`` (same draws, so x and the block's weights are a1's) and then,
    in this order: n ~ N(0,1) (what a LayerNorm of a random stream looks like; drawn, not computed: the
    generator holds no arithmetic of the method), gamma ~ N(1, 0.02) and beta ~ N(0, 0.02) of the middle
    LayerNorm, W1 ~ U(+-1/sqrt(C)), b1 likewise, W2 ~ U(+-1/sqrt(F)), b2 likewise, gamma and beta of the
    last LayerNorm.  F defaults to 4 C."""
    apb = make_attention(name, seed, **kw)
    B, T, C = apb.x.shape
    F = 4 * C if F is None else F
    rng = np.random.default_rng(seed + 1000)
    s = lambda a: _store(a, apb.dtype)
    n = s(_normal(rng, (B, T, C)))
    g_mid = s(_normal(rng, (C,), 1.0, 0.02)); be_mid = s(_normal(rng, (C,), 0.0, 0.02))
    w1 = s(_uniform(rng, (F, C), 1 / math.sqrt(C))); b1 = s(_uniform(rng, (F,), 1 / math.sqrt(C)))
    w2 = s(_uniform(rng, (C, F), 1 / math.sqrt(F))); b2 = s(_uniform(rng, (C,), 1 / math.sqrt(F)))
    g_out = s(_normal(rng, (C,), 1.0, 0.02)); be_out = s(_normal(rng, (C,), 0.0, 0.02))
    return LayerProblem(apb, n, g_mid, be_mid, w1, b1, w2, b2, g_out, be_out)


def make_qkv(seed: int, B: int, T: int, H: int, D: int, dtype: torch.dtype, spread: float = 1.0):
    """q, k, v for the attention kernel alone: one [B, T, 3, H, D] tensor ~ N(0, spread) (the layout a
    fused QKV projection writes); q, k, v are its views [:, :, i]."""
    rng = np.random.default_rng(seed)
    return _store(_normal(rng, (B, T, 3, H, D), 0.0, spread), dtype)


def to_f64(t):
    """Exact upcast of a stored tensor to a float64 numpy array (None passes through)."""
    return None if t is None else t.detach().cpu().to(torch.float64).numpy()


def epilogue_f64(epilogue, rows=None):
    """The epilogue list with its tensors upcast exactly to float64 numpy arrays.
    ``rows`` selects rows of [M,N] operands (every op is row-local)."""
    out = []
    for e in epilogue:
        if e[0] == "residual":
            r = e[1] if rows is None else e[1][rows]
            out.append(("residual", to_f64(r)))
        elif e[0] == "layernorm":
            out.append(("layernorm", to_f64(e[1]), to_f64(e[2]), e[3]))
        elif e[0] == "store":   # a fresh float64 target of the selected rows; the caller reads it back from the list
            t = e[1] if rows is None else e[1][rows]
            out.append(("store", np.full(tuple(t.shape), np.nan, dtype=np.float64)))
        else:
            out.append(tuple(e))
    return out
