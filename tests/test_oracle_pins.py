"""Pins for the CPU oracle: it is checked against what the mathematics fixes
(closed forms, tabulated values, invariants, brute force with exact rational
arithmetic) and against independent library routines (numpy, scipy, torch
CPU float64) -- never against itself and never against the GPU path.

The gold side of the paper's comparison is the original eager composition
(Appendix A, Correctness); the last group of tests pins exactly that.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch
import torch.nn.functional as F

import oracle

RNG = np.random.default_rng(1234)


def run(x, w, b=None, ep=()):
    return oracle.fused_linear_epilogue(np.asarray(x, np.float64), np.asarray(w, np.float64),
                                        None if b is None else np.asarray(b, np.float64), list(ep))


def elementwise(kind, v, *args):
    """Apply one op to a vector through the oracle: x = v as a column, W = [[1]]... i.e. K = 1."""
    v = np.asarray(v, np.float64).reshape(-1, 1)
    return run(v, np.ones((1, 1)), None, [(kind, *args)]).reshape(-1)


def rowop(ep, z):
    """Apply a chain to given rows z[M,N] through the oracle: W = identity."""
    z = np.asarray(z, np.float64)
    return run(z, np.eye(z.shape[1]), None, ep)


# ---------------------------------------------------------------- contraction
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 5), (3, 2, 8), (5, 17, 3), (8, 5, 17), (17, 8, 2)])
def test_contraction_brute_force_exact_rationals(M, N, K):
    x = RNG.standard_normal((M, K)); w = RNG.standard_normal((N, K))
    got = run(x, w)
    for m in range(M):
        for n in range(N):
            exact = sum(Fraction(float(x[m, k])) * Fraction(float(w[n, k])) for k in range(K))
            scale = sum(abs(float(x[m, k]) * float(w[n, k])) for k in range(K))
            assert abs(Fraction(float(got[m, n])) - exact) <= Fraction(1e-15) * Fraction(scale) * K


def test_contraction_is_x_times_w_transposed_not_w():
    # a non-square, asymmetric case with a known answer: catches a transposed operand
    x = np.array([[1.0, 2.0, 3.0]])
    w = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 0.0], [1.0, 1.0, 1.0], [0.0, 0.0, -2.0]])
    assert run(x, w).tolist() == [[1.0, 2.0, 6.0, -6.0]]


def test_contraction_special_operands():
    x = RNG.standard_normal((6, 9))
    assert np.array_equal(run(x, np.eye(9)), x)                      # W = I
    w = RNG.standard_normal((4, 9))
    e = np.zeros((1, 9)); e[0, 5] = 1.0
    assert np.array_equal(run(e, w)[0], w[:, 5])                     # one-hot row selects a column of W^T
    assert np.array_equal(run(np.ones((3, 40)), np.ones((2, 40))), np.full((3, 2), 40.0))


def test_contraction_small_integers_exact():
    x = RNG.integers(-2, 3, (13, 31)).astype(np.float64)
    w = RNG.integers(-2, 3, (7, 31)).astype(np.float64)
    want = (x.astype(np.int64) @ w.astype(np.int64).T).astype(np.float64)
    assert np.array_equal(run(x, w), want)


def test_contraction_vs_numpy_and_torch():
    x = RNG.standard_normal((33, 257)); w = RNG.standard_normal((65, 257))
    got = run(x, w)
    np.testing.assert_allclose(got, x @ w.T, rtol=0, atol=1e-11)
    np.testing.assert_allclose(got, F.linear(torch.from_numpy(x), torch.from_numpy(w)).numpy(), rtol=0, atol=1e-11)


def test_empty_and_degenerate_shapes():
    assert run(np.zeros((0, 4)), np.ones((3, 4))).shape == (0, 3)
    assert np.array_equal(run(np.zeros((2, 0)), np.zeros((3, 0)), np.array([1.0, 2.0, 3.0]), [("bias",)]),
                          np.array([[1.0, 2.0, 3.0]] * 2))           # K = 0: empty sum is 0


# ---------------------------------------------------------------- elementwise ops
def test_bias_scale_relu_residual_definitions():
    x = np.array([[1.0, -2.0], [0.5, 4.0]]); w = np.eye(2)
    assert run(x, w, [10.0, 20.0], [("bias",)]).tolist() == [[11.0, 18.0], [10.5, 24.0]]
    assert run(x, w, None, [("scale", -3.0)]).tolist() == [[-3.0, 6.0], [-1.5, -12.0]]
    assert run(x, w, None, [("relu",)]).tolist() == [[1.0, 0.0], [0.5, 4.0]]
    r = np.array([[100.0, 200.0], [300.0, 400.0]])
    assert run(x, w, None, [("residual", r)]).tolist() == [[101.0, 198.0], [300.5, 404.0]]
    out = elementwise("relu", [np.nan, -np.inf, np.inf, -0.0])
    assert np.isnan(out[0]) and out[1] == 0.0 and out[2] == np.inf and out[3] == 0.0


def _golden(name):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    return {float(a): float(b) for a, b in rows}


# Standard normal CDF table values (Phi): GELU-erf is x * Phi(x).
PHI = _golden("normal_cdf_points.txt")


def test_gelu_erf_fixed_points():
    xs = np.array([0.0, 0.5, -0.5, 1.0, -1.0, 2.0, 3.0, -3.0])
    want = np.array([0.0, 0.5 * PHI[0.5], -0.5 * (1 - PHI[0.5]), PHI[1.0], -(1 - PHI[1.0]),
                     2 * PHI[2.0], 3 * PHI[3.0], -3 * (1 - PHI[3.0])])
    np.testing.assert_allclose(elementwise("gelu_erf", xs), want, rtol=0, atol=2e-15)


def test_gelu_erf_vs_scipy_cdf_and_oddness():
    xs = np.linspace(-8, 8, 4001)
    g = elementwise("gelu_erf", xs)
    np.testing.assert_allclose(g, xs * scipy.stats.norm.cdf(xs), rtol=0, atol=1e-14)
    np.testing.assert_allclose(g - elementwise("gelu_erf", -xs), xs, rtol=0, atol=1e-14)   # g(x) - g(-x) = x


def test_gelu_tanh_fixed_points_and_library():
    # values of 0.5 x (1 + tanh(sqrt(2/pi)(x + 0.044715 x^3))) worked out with mpmath-grade arithmetic
    pts = _golden("gelu_tanh_points.txt")
    xs = np.array(sorted(pts)); want = np.array([pts[x] for x in sorted(pts)])
    np.testing.assert_allclose(elementwise("gelu_tanh", xs), want, rtol=0, atol=2e-15)
    grid = np.linspace(-6, 6, 2401)
    g = elementwise("gelu_tanh", grid)
    np.testing.assert_allclose(g, F.gelu(torch.from_numpy(grid), approximate="tanh").numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(g - elementwise("gelu_tanh", -grid), grid, rtol=0, atol=1e-14)
    # the two GELU variants differ, by at most 4.73e-4 (near |x| = 2.7): a swapped variant is detectable
    d = np.abs(g - elementwise("gelu_erf", grid))
    assert 4.6e-4 < d.max() < 4.8e-4 and 2.5 < abs(grid[d.argmax()]) < 2.9


# ---------------------------------------------------------------- row ops
def test_layernorm_closed_forms():
    z = RNG.standard_normal((5, 64)) * 3 + 7
    eps = 1e-5
    y = rowop([("layernorm", None, None, eps)], z)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-13)
    var = z.var(axis=1)                                # biased
    epsf = float(np.float32(eps))
    np.testing.assert_allclose(y.var(axis=1), var / (var + epsf), rtol=1e-12)   # not 1: eps sits inside the sqrt
    # constant row -> beta; N = 1 -> beta
    beta = RNG.standard_normal(64); gamma = RNG.standard_normal(64)
    yc = rowop([("layernorm", gamma, beta, eps)], np.full((2, 64), 3.25))
    np.testing.assert_allclose(yc, np.tile(beta, (2, 1)), atol=1e-15)
    assert rowop([("layernorm", np.array([2.0]), np.array([-7.0]), eps)], [[5.0]]).tolist() == [[-7.0]]
    # affine invariance at eps = 0, and the affine step comes after normalisation
    y0 = rowop([("layernorm", None, None, 0.0)], z)
    np.testing.assert_allclose(rowop([("layernorm", None, None, 0.0)], 2.5 * z - 4), y0, atol=1e-12)
    np.testing.assert_allclose(rowop([("layernorm", gamma, beta, 0.0)], z), y0 * gamma + beta, atol=1e-13)


def test_layernorm_hand_example_and_torch():
    # row (1,2,3,4): mean 2.5, biased variance 1.25
    y = rowop([("layernorm", None, None, 0.0)], [[1.0, 2.0, 3.0, 4.0]])
    np.testing.assert_allclose(y[0], np.array([-1.5, -0.5, 0.5, 1.5]) / math.sqrt(1.25), atol=1e-15)
    z = RNG.standard_normal((7, 96)); g = RNG.standard_normal(96); be = RNG.standard_normal(96)
    eps = float(np.float32(1e-5))
    want = F.layer_norm(torch.from_numpy(z), (96,), torch.from_numpy(g), torch.from_numpy(be), eps).numpy()
    np.testing.assert_allclose(rowop([("layernorm", g, be, 1e-5)], z), want, atol=1e-12)


def test_softmax_closed_forms():
    z = RNG.standard_normal((6, 50)) * 4
    s = rowop([("softmax",)], z)
    np.testing.assert_allclose(s.sum(axis=1), 1, atol=1e-14)
    assert (s > 0).all() and (s <= 1).all()
    np.testing.assert_allclose(rowop([("softmax",)], z + 123.0), s, atol=1e-13)       # shift invariance
    np.testing.assert_allclose(s, scipy.special.softmax(z, axis=1), atol=1e-15)
    two = rowop([("softmax",)], [[0.3, -1.1]])
    assert abs(two[0, 0] - 1 / (1 + math.exp(-1.4))) < 1e-15                          # N = 2 is the logistic
    np.testing.assert_allclose(rowop([("softmax",)], np.full((1, 8), -3.0)), 0.125, atol=1e-16)
    big = rowop([("softmax",)], [[1000.0, 1000.0, -1000.0]])                          # no overflow
    np.testing.assert_allclose(big, [[0.5, 0.5, 0.0]], atol=1e-300)


def test_logsumexp_closed_forms():
    z = RNG.standard_normal((6, 50)) * 4
    l = rowop([("logsumexp",)], z)
    assert l.shape == (6,)
    np.testing.assert_allclose(l, np.log(np.exp(z).sum(axis=1)), atol=1e-13)          # the definition, |z| small
    np.testing.assert_allclose(rowop([("logsumexp",)], z + 77.0), l + 77.0, atol=1e-12)
    np.testing.assert_allclose(rowop([("logsumexp",)], np.full((1, 32), 2.0)), 2.0 + math.log(32), atol=1e-15)
    np.testing.assert_allclose(l, scipy.special.logsumexp(z, axis=1), atol=1e-13)
    np.testing.assert_allclose(np.exp(z - l[:, None]), rowop([("softmax",)], z), atol=1e-14)  # ties both ops
    assert rowop([("logsumexp",)], [[1000.0, 1000.0]])[0] == pytest.approx(1000.0 + math.log(2), abs=1e-12)


# ---------------------------------------------------------------- composition and order
def test_order_matters():
    x = np.array([[2.0, -3.0]]); w = np.eye(2)
    assert run(x, w, None, [("scale", -1.0), ("relu",)]).tolist() == [[0.0, 3.0]]
    assert run(x, w, None, [("relu",), ("scale", -1.0)]).tolist() == [[-2.0, 0.0]]
    b = [-2.5, 4.0]
    assert run(x, w, b, [("bias",), ("relu",)]).tolist() == [[0.0, 1.0]]
    assert run(x, w, b, [("relu",), ("bias",)]).tolist() == [[-0.5, 4.0]]
    # a row op in the middle of the list, then an elementwise op
    got = run(x, w, None, [("softmax",), ("scale", 2.0)])
    np.testing.assert_allclose(got, 2 * scipy.special.softmax(x, axis=1), atol=1e-15)


def torch_eager(x, w, b, ep):
    """The unfused PyTorch-eager composition in float64 on the CPU."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    z = F.linear(t(x), t(w))
    for e in ep:
        k = e[0]
        if k == "bias": z = z + t(b)
        elif k == "scale": z = z * float(np.float32(e[1]))
        elif k == "relu": z = F.relu(z)
        elif k == "gelu_erf": z = F.gelu(z)
        elif k == "gelu_tanh": z = F.gelu(z, approximate="tanh")
        elif k == "residual": z = z + t(e[1])
        elif k == "layernorm":
            z = F.layer_norm(z, (z.shape[1],), None if e[1] is None else t(e[1]),
                             None if e[2] is None else t(e[2]), float(np.float32(e[3])))
        elif k == "softmax": z = torch.softmax(z, -1)
        elif k == "logsumexp": z = torch.logsumexp(z, -1)
    return z.numpy()


CHAINS = [
    ["bias", "gelu_erf"],
    ["bias", "relu", "scale", "residual"],
    ["bias", "gelu_tanh", "layernorm"],
    ["softmax"],
    ["bias", "residual", "layernorm"],
    ["scale", "logsumexp"],
    ["bias", "layernorm", "gelu_erf", "residual"],
    ["relu", "softmax", "scale"],
    ["layernorm", "softmax"],
    ["bias", "gelu_tanh", "scale", "relu", "residual", "logsumexp"],
]


@pytest.mark.parametrize("kinds", CHAINS)
def test_composition_matches_torch_cpu_float64(kinds):
    M, N, K = 9, 40, 23
    x = RNG.standard_normal((M, K)); w = RNG.standard_normal((N, K)) / 4; b = RNG.standard_normal(N)
    ep = []
    for k in kinds:
        if k == "scale": ep.append(("scale", 0.7))
        elif k == "residual": ep.append(("residual", RNG.standard_normal((M, N))))
        elif k == "layernorm": ep.append(("layernorm", RNG.standard_normal(N), RNG.standard_normal(N), 1e-5))
        else: ep.append((k,))
    np.testing.assert_allclose(run(x, w, b, ep), torch_eager(x, w, b, ep), rtol=1e-11, atol=1e-11)


def test_structural_invariants():
    M, N, K = 12, 24, 16
    x = RNG.standard_normal((M, K)); w = RNG.standard_normal((N, K)) / 4; b = RNG.standard_normal(N)
    r = RNG.standard_normal((M, N)); g = RNG.standard_normal(N); be = RNG.standard_normal(N)
    ep = lambda r_, g_, be_: [("bias",), ("gelu_tanh",), ("residual", r_), ("layernorm", g_, be_, 1e-5)]
    base = run(x, w, b, ep(r, g, be))
    pm = RNG.permutation(M); pn = RNG.permutation(N)
    np.testing.assert_allclose(run(x[pm], w, b, ep(r[pm], g, be)), base[pm], atol=1e-13)          # rows
    np.testing.assert_allclose(run(x, w[pn], b[pn], ep(r[:, pn], g[pn], be[pn])), base[:, pn], atol=1e-12)  # columns
    xz = np.hstack([x, np.zeros((M, 32))]); wz = np.hstack([w, RNG.standard_normal((N, 32))])
    np.testing.assert_allclose(run(xz, wz, b, ep(r, g, be)), base, atol=1e-13)                    # zero K padding
    top = run(x[:5], w, b, ep(r[:5], g, be)); bot = run(x[5:], w, b, ep(r[5:], g, be))
    assert np.array_equal(np.vstack([top, bot]), base)                                            # split M


def test_store_copies_the_values_at_its_place_in_the_chain():
    M, N, K = 5, 7, 3
    x, w, b, r = RNG.standard_normal((M, K)), RNG.standard_normal((N, K)), RNG.standard_normal(N), RNG.standard_normal((M, N))
    g, be = RNG.standard_normal(N), RNG.standard_normal(N)
    t1, t2, t3 = (np.full((M, N), np.nan) for _ in range(3))
    out = run(x, w, b, [("store", t1), ("bias",), ("residual", r), ("store", t2), ("layernorm", g, be, 1e-5), ("store", t3), ("relu",)])
    # each copy equals the chain cut off at that point, and the chain's own result is what it is without the stores
    np.testing.assert_array_equal(t1, run(x, w, b, []))
    np.testing.assert_array_equal(t2, run(x, w, b, [("bias",), ("residual", r)]))
    np.testing.assert_array_equal(t3, run(x, w, b, [("bias",), ("residual", r), ("layernorm", g, be, 1e-5)]))
    np.testing.assert_array_equal(out, run(x, w, b, [("bias",), ("residual", r), ("layernorm", g, be, 1e-5), ("relu",)]))
    # independent values: t2 is x w^T + b + r by numpy
    np.testing.assert_allclose(t2, x @ w.T + b + r, rtol=1e-13, atol=1e-13)
    with pytest.raises(ValueError):
        run(x, w, b, [("store", np.zeros((M, N + 1)))])


def test_rejects_bad_arguments():
    x = np.zeros((2, 3)); w = np.zeros((4, 3))
    with pytest.raises(ValueError):
        run(x, w, None, [("bias",)])                      # bias op without b
    with pytest.raises(ValueError):
        run(x, w, None, [("logsumexp",), ("relu",)])      # logsumexp must be last
    with pytest.raises(TypeError):
        oracle.fused_linear_epilogue(x.astype(np.float32), w, None, [])


# ---------------------------------------------------------------- grouped form
def grouped(x, w, b, offsets, ep=()):
    return oracle.grouped_fused_linear_epilogue(np.asarray(x, np.float64), np.asarray(w, np.float64),
                                                None if b is None else np.asarray(b, np.float64), offsets, list(ep))


def test_grouped_equals_one_hot_masked_sum():
    """Independent formulation (numpy only): out[m] = sum_g [m in group g] (x[m] W_g^T + b_g)."""
    counts = [3, 0, 5, 1, 0, 4]
    G, N, K = len(counts), 7, 6
    off = np.concatenate([[0], np.cumsum(counts)])
    M = int(off[-1])
    x = RNG.standard_normal((M, K)); w = RNG.standard_normal((G, N, K)); b = RNG.standard_normal((G, N))
    owner = np.repeat(np.arange(G), counts)
    onehot = (owner[:, None] == np.arange(G)[None, :]).astype(np.float64)     # [M, G]
    dense = np.einsum("mk,gnk->mgn", x, w) + b[None, :, :]                      # every row through every group
    want = np.einsum("mg,mgn->mn", onehot, dense)
    np.testing.assert_allclose(grouped(x, w, b, off, [("bias",)]), want, atol=1e-13)
    # a group index shifted by one, a transposed W_g or a dropped bias would all differ
    assert np.abs(want - (np.einsum("mg,mgn->mn", np.roll(onehot, 1, axis=1), dense))).max() > 0.1
    # shared bias [N]
    np.testing.assert_allclose(grouped(x, w, b[0], off, [("bias",)]), np.einsum("mg,mgn->mn", onehot, np.einsum("mk,gnk->mgn", x, w)) + b[0], atol=1e-13)


def test_grouped_store_targets_follow_the_groups():
    """Independent formulation (numpy only): a store after bias and residual holds, in row m, x[m] W_g^T + b_g + r[m]
    of the group g that owns the row; rows of no group do not exist, so every element is written."""
    counts = [2, 0, 4, 3]
    off = np.concatenate([[0], np.cumsum(counts)])
    M, N, K = int(off[-1]), 6, 5
    x = RNG.standard_normal((M, K)); w = RNG.standard_normal((4, N, K)); b = RNG.standard_normal((4, N)); r = RNG.standard_normal((M, N))
    t = np.full((M, N), np.nan)
    out = grouped(x, w, b, off, [("bias",), ("residual", r), ("store", t), ("relu",)])
    owner = np.repeat(np.arange(4), counts)
    want = np.einsum("mk,mnk->mn", x, w[owner]) + b[owner] + r
    np.testing.assert_allclose(t, want, atol=1e-13)
    np.testing.assert_allclose(out, np.maximum(want, 0.0), atol=1e-13)
    assert np.abs(want - (np.einsum("mk,mnk->mn", x, w[np.roll(owner, 1)]) + b[owner] + r)).max() > 0.1   # a shifted owner differs


def test_grouped_reductions_and_plain_form():
    counts = [4, 2, 6]
    off = [0, 4, 6, 12]
    M, N, K = 12, 10, 5
    x = RNG.standard_normal((M, K)); w = RNG.standard_normal((3, N, K)); b = RNG.standard_normal((3, N))
    r = RNG.standard_normal((M, N)); g = RNG.standard_normal(N); be = RNG.standard_normal(N)
    ep = [("bias",), ("gelu_tanh",), ("residual", r), ("layernorm", g, be, 1e-5)]
    got = grouped(x, w, b, off, ep)
    # every row equals the plain operator applied to that row alone with its group's weights
    for m in range(M):
        gi = 0 if m < 4 else 1 if m < 6 else 2
        one = run(x[m:m + 1], w[gi], b[gi], [("bias",), ("gelu_tanh",), ("residual", r[m:m + 1]), ("layernorm", g, be, 1e-5)])
        assert np.array_equal(got[m], one[0])
    # one group is the plain form; equal weights in every group are the plain form too
    assert np.array_equal(grouped(x, w[:1], b[:1], [0, M], ep), run(x, w[0], b[0], ep))
    same = np.stack([w[1]] * 3); sb = np.stack([b[1]] * 3)
    assert np.array_equal(grouped(x, same, sb, off, ep), run(x, w[1], b[1], ep))
    # logsumexp gives one value per row; empty groups change nothing
    lse = grouped(x, w, b, off, [("bias",), ("logsumexp",)])
    assert lse.shape == (M,)
    np.testing.assert_allclose(lse[4:6], scipy.special.logsumexp(x[4:6] @ w[1].T + b[1], axis=1), atol=1e-12)
    w5 = np.stack([w[0], w[2], w[1], w[0], w[2]]); b5 = np.stack([b[0], b[2], b[1], b[0], b[2]])
    assert np.array_equal(grouped(x, w5, b5, [0, 4, 4, 6, 6, 12], ep), got)
    # swapping two groups' row blocks together with their weights permutes the output blocks
    perm = np.concatenate([np.arange(6, 12), np.arange(4, 6), np.arange(0, 4)])
    sw = grouped(x[perm], w[[2, 1, 0]], b[[2, 1, 0]], [0, 6, 8, 12], [("bias",), ("gelu_tanh",), ("residual", r[perm]), ("layernorm", g, be, 1e-5)])
    assert np.array_equal(sw, got[perm])


def test_grouped_rejects_bad_offsets():
    x = np.zeros((4, 3)); w = np.zeros((2, 5, 3))
    for off in ([0, 2], [0, 3, 2], [1, 2, 4], [0, 2, 5], [0, 3, 2, 4]):
        with pytest.raises(ValueError):
            grouped(x, w, None, off)
    assert grouped(x, w, None, [0, 0, 4]).shape == (4, 5)


# ------------------------------------------------------------------ attention (the block the paper's
# task-wise analysis names as its largest recurring win; appendix on Level 3-pike / Level 5 outliers)
def _qkv(B, T, H, D, rng=RNG):
    return tuple(rng.standard_normal((B, T, H, D)) for _ in range(3))


def test_attention_closed_forms():
    B, T, H, D = 2, 9, 3, 4
    q, k, v = _qkv(B, T, H, D)
    # causal: the first query sees one key, so its output is that key's value row
    o = oracle.attention(q, k, v, True)
    np.testing.assert_allclose(o[:, 0], v[:, 0], rtol=0, atol=1e-15)
    # equal scores (q = 0, or all keys equal): uniform weights -> (prefix) mean of v
    o = oracle.attention(np.zeros_like(q), k, v, False)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape), rtol=0, atol=1e-14)
    same_k = np.broadcast_to(k[:, :1], k.shape).copy()
    o = oracle.attention(q, same_k, v, True)
    prefix_mean = np.cumsum(v, axis=1) / np.arange(1, T + 1).reshape(1, T, 1, 1)
    np.testing.assert_allclose(o, prefix_mean, rtol=0, atol=1e-14)
    # two keys, D = 4 (default scale 1/2): weights are the logistic function of the score difference
    q2 = np.zeros((1, 2, 1, 4)); k2 = np.zeros((1, 2, 1, 4)); v2 = np.zeros((1, 2, 1, 4))
    q2[0, :, 0, 0] = [2.0, -6.0]
    k2[0, 0, 0, 0] = 1.0
    v2[0, 0, 0] = [1, 0, 3, 0]; v2[0, 1, 0] = [0, 1, 0, -2]
    o = oracle.attention(q2, k2, v2, False)
    s1 = 0.7310585786300049  # 1 / (1 + e^-1): query 0 scores (1, 0)
    np.testing.assert_allclose(o[0, 0, 0], s1 * v2[0, 0, 0] + (1 - s1) * v2[0, 1, 0], rtol=0, atol=1e-15)
    s3 = 1.0 / (1.0 + math.exp(3.0))  # query 1 scores (-3, 0)
    np.testing.assert_allclose(o[0, 1, 0], s3 * v2[0, 0, 0] + (1 - s3) * v2[0, 1, 0], rtol=0, atol=1e-15)
    # an explicit scale: zero makes the weights uniform again
    o = oracle.attention(q, k, v, False, scale=0.0)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape), rtol=0, atol=1e-14)


def test_attention_selects_the_matching_key():
    # keys are far-apart one-hot rows and query t points at key perm[t]: the weights collapse onto it
    T, D = 6, 8
    perm = np.array([3, 0, 5, 1, 4, 2])
    k = np.zeros((1, T, 1, D)); q = np.zeros((1, T, 1, D))
    for j in range(T):
        k[0, j, 0, j] = 40.0
        q[0, j, 0, perm[j]] = 40.0
    v = RNG.standard_normal((1, T, 1, D))
    o = oracle.attention(q, k, v, False)
    np.testing.assert_allclose(o[0, :, 0], v[0, perm, 0], rtol=0, atol=1e-12)


def test_attention_invariants():
    B, T, H, D = 2, 11, 2, 8
    q, k, v = _qkv(B, T, H, D)
    base = oracle.attention(q, k, v, False)
    # no mask: the order of the keys does not matter; permuting queries permutes outputs
    perm = RNG.permutation(T)
    np.testing.assert_allclose(oracle.attention(q, k[:, perm], v[:, perm], False), base, rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.attention(q[:, perm], k, v, False), base[:, perm], rtol=0, atol=1e-14)
    # a vector added to every key shifts all of a query's scores alike
    c = RNG.standard_normal((1, 1, H, D))
    np.testing.assert_allclose(oracle.attention(q, k + c, v, False), base, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.attention(q, k + c, v, True), oracle.attention(q, k, v, True), rtol=0, atol=1e-13)
    # heads and batch entries are independent problems
    alone = oracle.attention(q[1:, :, 1:], k[1:, :, 1:], v[1:, :, 1:], True)
    np.testing.assert_allclose(oracle.attention(q, k, v, True)[1:, :, 1:], alone, rtol=0, atol=0)
    # causal: outputs up to t do not depend on later tokens
    cut = 5
    np.testing.assert_allclose(oracle.attention(q, k, v, True)[:, :cut],
                               oracle.attention(q[:, :cut], k[:, :cut], v[:, :cut], True), rtol=0, atol=0)
    # evaluating only the last queries gives the same rows
    for causal in (False, True):
        np.testing.assert_allclose(oracle.attention(q, k, v, causal, first_query=7), oracle.attention(q, k, v, causal)[:, 7:], rtol=0, atol=0)
    # linear in v; outputs are convex combinations of the value rows
    np.testing.assert_allclose(oracle.attention(q, k, 2 * v + 1, False), 2 * base + 1, rtol=0, atol=1e-13)
    assert (base <= v.max(axis=1, keepdims=True) + 1e-14).all() and (base >= v.min(axis=1, keepdims=True) - 1e-14).all()


@pytest.mark.parametrize("causal", [False, True])
def test_attention_matches_torch_cpu_float64(causal):
    B, T, H, D = 2, 13, 3, 16
    q, k, v = _qkv(B, T, H, D)
    tq, tk, tv = (torch.from_numpy(a).permute(0, 2, 1, 3) for a in (q, k, v))  # torch wants [B,H,T,D]
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=float(np.float32(1 / math.sqrt(D))))
    np.testing.assert_allclose(oracle.attention(q, k, v, causal), ref.permute(0, 2, 1, 3).numpy(), rtol=1e-12, atol=1e-13)
    # views into one fused [B,T,3,H,D] buffer are accepted as they are
    qkv = np.stack([q, k, v], axis=2)
    np.testing.assert_allclose(oracle.attention(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], causal),
                               oracle.attention(q, k, v, causal), rtol=0, atol=0)


def test_attention_block_layout_and_composition():
    B, T, C, heads = 2, 6, 8, 2
    D = C // heads
    x = RNG.standard_normal((B, T, C))
    # q and k thirds zero, v third and output projection the identity: causal prefix mean of x
    w_qkv = np.zeros((3 * C, C)); w_qkv[2 * C:] = np.eye(C)
    b_o = RNG.standard_normal(C); res = RNG.standard_normal((B, T, C))
    y = oracle.attention_block(x, w_qkv, None, np.eye(C), b_o, heads, True, residual=res)
    prefix_mean = np.cumsum(x, axis=1) / np.arange(1, T + 1).reshape(1, T, 1)
    np.testing.assert_allclose(y, prefix_mean + b_o + res, rtol=0, atol=1e-14)
    # column layout of the projection's output is [q | k | v], each cut into heads of D columns:
    # against the same block composed from torch CPU float64 ops
    w_qkv = RNG.standard_normal((3 * C, C)) * 0.5; b_qkv = RNG.standard_normal(3 * C)
    w_o = RNG.standard_normal((C, C)) * 0.5
    tx = torch.from_numpy(x)
    qkv = F.linear(tx, torch.from_numpy(w_qkv), torch.from_numpy(b_qkv))
    tq, tk, tv = (t.reshape(B, T, heads, D).transpose(1, 2) for t in qkv.split(C, dim=2))
    att = F.scaled_dot_product_attention(tq, tk, tv, is_causal=False, scale=float(np.float32(1 / math.sqrt(D))))
    ref = F.linear(att.transpose(1, 2).reshape(B, T, C), torch.from_numpy(w_o), torch.from_numpy(b_o))
    y = oracle.attention_block(x, w_qkv, b_qkv, w_o, b_o, heads, False)
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)
    # heads differ: with a single head over all C columns the result changes
    assert np.abs(oracle.attention_block(x, w_qkv, b_qkv, w_o, b_o, 1, False) - y).max() > 1e-3


def test_attention_group_causal_mask():
    B, T, H, D = 2, 23, 2, 8
    q, k, v = _qkv(B, T, H, D)
    # groups of one token are the plain causal mask; one group holding the whole sequence is no mask
    np.testing.assert_allclose(oracle.attention(q, k, v, 1), oracle.attention(q, k, v, True), rtol=0, atol=0)
    for G in (T, T + 5):
        np.testing.assert_allclose(oracle.attention(q, k, v, G), oracle.attention(q, k, v, False), rtol=0, atol=0)
    for G in (2, 5, 8):
        limit = np.minimum(T, (np.arange(T) // G + 1) * G)             # keys visible to query t: 0 .. limit[t] - 1
        # equal scores: the mean of the visible value rows
        o = oracle.attention(np.zeros_like(q), k, v, G)
        want = np.stack([v[:, :limit[t]].mean(axis=1) for t in range(T)], axis=1)
        np.testing.assert_allclose(o, want, rtol=0, atol=1e-14)
        # against torch CPU float64 with the mask spelt out
        mask = torch.from_numpy(np.arange(T)[None, :] < limit[:, None])
        tq, tk, tv = (torch.from_numpy(a).permute(0, 2, 1, 3) for a in (q, k, v))
        ref = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=float(np.float32(1 / math.sqrt(D))))
        np.testing.assert_allclose(oracle.attention(q, k, v, G), ref.permute(0, 2, 1, 3).numpy(), rtol=1e-12, atol=1e-13)
        # all queries of a group see the same keys, so permuting the keys inside a group changes nothing
        perm = np.arange(T); perm[:G] = perm[:G][::-1]
        np.testing.assert_allclose(oracle.attention(q, k[:, perm], v[:, perm], G), oracle.attention(q, k, v, G), rtol=0, atol=1e-14)


def test_attention_with_more_keys_than_queries():
    B, T, Tk, H, D = 2, 5, 12, 2, 8
    q, _, _ = _qkv(B, T, H, D)
    _, k, v = _qkv(B, Tk, H, D)
    # no mask: each query is its own problem, so any subset of the queries of a square problem agrees with it
    qq = RNG.standard_normal((B, Tk, H, D))
    full = oracle.attention(qq, k, v, False)
    np.testing.assert_allclose(oracle.attention(qq[:, 3:8], k, v, False), full[:, 3:8], rtol=0, atol=0)
    # causal: the queries are the last T positions, so they equal the last T rows of the square causal problem
    full = oracle.attention(qq, k, v, True)
    np.testing.assert_allclose(oracle.attention(qq[:, Tk - T:], k, v, True), full[:, Tk - T:], rtol=0, atol=0)
    for G in (3, 4):
        full = oracle.attention(qq, k, v, G)
        np.testing.assert_allclose(oracle.attention(qq[:, Tk - T:], k, v, G), full[:, Tk - T:], rtol=0, atol=0)
    # equal scores: mean of the visible values; the first of the T queries stands at position Tk - T
    o = oracle.attention(np.zeros((B, T, H, D)), k, v, True)
    want = np.stack([v[:, :Tk - T + t + 1].mean(axis=1) for t in range(T)], axis=1)
    np.testing.assert_allclose(o, want, rtol=0, atol=1e-14)
    # against torch CPU float64 with the mask spelt out (one query, the decoding case, included)
    for Tq in (1, T):
        qs = q[:, :Tq]
        mask = torch.from_numpy(np.arange(Tk)[None, :] <= (np.arange(Tq) + Tk - Tq)[:, None])
        tq, tk, tv = (torch.from_numpy(a).permute(0, 2, 1, 3) for a in (qs, k, v))
        ref = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=float(np.float32(1 / math.sqrt(D))))
        np.testing.assert_allclose(oracle.attention(qs, k, v, True), ref.permute(0, 2, 1, 3).numpy(), rtol=1e-12, atol=1e-13)
    with pytest.raises(ValueError):
        oracle.attention(qq, k[:, :4], v[:, :4], True)        # causal with fewer keys than queries


def test_attention_rejects_bad_arguments():
    q, k, v = _qkv(1, 3, 1, 4)
    with pytest.raises(ValueError):
        oracle.attention(q, k[:, :2], v, False)                  # k and v differ in length
    with pytest.raises(TypeError):
        oracle.attention(q.astype(np.float32), k, v, False)
    with pytest.raises(ValueError):
        oracle.attention_block(np.zeros((1, 2, 6)), np.zeros((18, 6)), None, np.eye(6), None, 4, False)


def test_transformer_layer_against_a_numpy_formulation():
    """The pre-norm layer from its normalised input on, written independently: per sequence and head an
    explicit masked softmax in numpy, LayerNorm from numpy's mean and variance, GELU from scipy's erf."""
    B, T, C, heads, Fh = 2, 7, 12, 3, 20
    D = C // heads
    x = RNG.standard_normal((B, T, C)); n = RNG.standard_normal((B, T, C))
    w_qkv = RNG.standard_normal((3 * C, C)) * 0.4; b_qkv = RNG.standard_normal(3 * C) * 0.1
    w_o = RNG.standard_normal((C, C)) * 0.4; b_o = RNG.standard_normal(C) * 0.1
    w1 = RNG.standard_normal((Fh, C)) * 0.4; b1 = RNG.standard_normal(Fh) * 0.1
    w2 = RNG.standard_normal((C, Fh)) * 0.4; b2 = RNG.standard_normal(C) * 0.1
    g1, be1, g2, be2 = (RNG.standard_normal(C) for _ in range(4))
    eps = 1e-5

    def ln(a, g, be):
        mu = a.mean(axis=-1, keepdims=True); var = ((a - mu) ** 2).mean(axis=-1, keepdims=True)
        return (a - mu) / np.sqrt(var + np.float64(np.float32(eps))) * g + be

    for causal in (True, False):
        got_x, got_n = oracle.transformer_layer(x, n, w_qkv, b_qkv, w_o, b_o, heads, causal, (g1, be1, eps), w1, b1, w2, b2, (g2, be2, eps))
        qkv = n @ w_qkv.T + b_qkv
        att = np.zeros((B, T, C))
        scale = np.float64(np.float32(1 / math.sqrt(D)))
        for b in range(B):
            for hd in range(heads):
                q = qkv[b, :, hd * D:(hd + 1) * D]; k = qkv[b, :, C + hd * D:C + (hd + 1) * D]; v = qkv[b, :, 2 * C + hd * D:2 * C + (hd + 1) * D]
                s = q @ k.T * scale
                if causal:
                    s = np.where(np.arange(T)[None, :] <= np.arange(T)[:, None], s, -np.inf)
                p = np.exp(s - s.max(axis=1, keepdims=True)); p /= p.sum(axis=1, keepdims=True)
                att[b, :, hd * D:(hd + 1) * D] = p @ v
        h = x + att @ w_o.T + b_o
        m = ln(h, g1, be1)
        pre = m @ w1.T + b1
        want_x = h + (0.5 * pre * (1 + scipy.special.erf(pre / math.sqrt(2)))) @ w2.T + b2
        want_n = ln(want_x, g2, be2)
        np.testing.assert_allclose(got_x, want_x, rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(got_n, want_n, rtol=1e-10, atol=1e-10)
        # plausible mistakes differ: the perceptron added to x instead of h, or the middle LayerNorm taken of x
        assert np.abs(want_x - (x + (want_x - h))).max() > 1e-2
        assert np.abs(got_n - ln(h, g2, be2)).max() > 1e-2


def test_mx_dequantize_follows_the_e8m0_definition():
    """OCP Microscaling Formats specification: a scale byte e stands for 2^(e - 127), 255 for NaN, and it covers 32
    consecutive elements of its row.  The expected values are that definition evaluated by hand."""
    elems = np.ones((2, 96))
    elems[0, 31], elems[0, 32], elems[1, 95] = -3.0, 5.0, 0.5
    scales = np.array([[127, 128, 120], [0, 254, 255]], dtype=np.uint8)
    got = oracle.mx_dequantize(elems, scales)
    assert got.shape == (2, 96) and got.dtype == np.float64
    assert got[0, 0] == 1.0 and got[0, 31] == -3.0            # byte 127: the values themselves
    assert got[0, 32] == 10.0 and got[0, 63] == 2.0           # byte 128 starts exactly at element 32
    assert got[0, 64] == 0.0078125                            # byte 120: 2^-7
    assert got[1, 0] == 5.877471754111438e-39                 # byte 0: 2^-127
    assert got[1, 32] == 1.7014118346046923e38                # byte 254: 2^127
    assert np.isnan(got[1, 64:]).all() and not np.isnan(got[1, :64]).any()
    # a dot product of block-scaled rows is the plain one of the dequantised values
    w = oracle.mx_dequantize(np.full((1, 96), 2.0), np.array([[126, 127, 130]], dtype=np.uint8))
    y = oracle.fused_linear_epilogue(got[:1], w, None, [])
    assert y[0, 0] == (31 * 1.0 - 3.0) * 1.0 + (5.0 + 31) * 2.0 * 2.0 + 32 * 0.0078125 * 16.0 == 176.0   # w: 2 * 2^-1, 2 * 1, 2 * 2^3 per block
    with pytest.raises(ValueError):
        oracle.mx_dequantize(np.ones((2, 96)), np.zeros((2, 2), dtype=np.uint8))
    with pytest.raises(ValueError):
        oracle.mx_dequantize(np.ones((2, 96)), np.zeros((2, 3), dtype=np.int32))


def test_mx_quantize_round_trips_within_an_e4m3_rounding():
    """The input generator's quantiser against the oracle's decoder: every value comes back within one e4m3 rounding
    (2^-4 relative, or the subnormal step of the block's scale), powers of two are exact, and the scale is the one
    the specification's recipe gives."""
    from paper_2511_16964_amd import inputs
    rng = np.random.default_rng(3)
    a = rng.standard_normal((8, 256)) * np.ldexp(1.0, rng.integers(-10, 10, size=(8, 8))).repeat(32, axis=1)
    a[0, :32] = 0.0
    a[1, 32:64] = np.ldexp(1.0, np.arange(32) % 7)
    q, s = inputs.mx_quantize(a)
    back = oracle.mx_dequantize(q.to(torch.float64).numpy(), s.numpy())
    amax = np.abs(a).reshape(8, 8, 32).max(axis=2).repeat(32, axis=1)
    scale = np.ldexp(1.0, s.numpy().astype(np.int64) - 127).repeat(32, axis=1)
    near = np.abs(back - a) <= np.maximum(np.abs(a) * 2.0 ** -4, amax * 2.0 ** -10)
    saturated = (np.abs(a) > 448 * scale) & (back == np.sign(a) * 448 * scale)   # (the format's largest value is 1.75 * 2^8: a block maximum above 1.75 times its power of two is cut there)
    assert (near | saturated).all() and saturated.sum() < near.size // 20
    assert (amax[:, ::32][amax[:, ::32] > 0] >= 256 * scale[:, ::32][amax[:, ::32] > 0]).all() and (amax < 512 * scale)[amax > 0].all()   # e = floor(log2(max)) - 8
    assert (back[0, :32] == 0).all() and (back[1, 32:64] == a[1, 32:64]).all()
    assert s.dtype == torch.uint8 and s.shape == (8, 8) and s[0, 0] == 0


def test_layernorm_rows_matches_torch_and_the_row_op():
    """The LayerNorm that precedes the multiplication: against torch's CPU float64 layer_norm (a library routine with
    the same definition), against the oracle's own row op over N applied to x I^T (independent C code, pinned above),
    and on a row whose result is known in closed form."""
    rng = np.random.default_rng(11)
    x = rng.standard_normal((5, 48)) * 3.0 + 7.0
    g, b = rng.standard_normal(48), rng.standard_normal(48)
    got = oracle.layernorm_rows(x, g, b, 2.0 ** -10)   # (an eps that float32, in which the row op takes it, holds exactly)
    ref = F.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), 2.0 ** -10).numpy()
    assert np.abs(got - ref).max() < 1e-13
    via_row_op = oracle.fused_linear_epilogue(x, np.eye(48), None, [("layernorm", g, b, 2.0 ** -10)])
    assert np.abs(got - via_row_op).max() < 1e-13
    assert np.abs(oracle.layernorm_rows(x, None, None, 0.0).mean(axis=1)).max() < 1e-14
    assert np.abs(oracle.layernorm_rows(x, None, None, 0.0).var(axis=1) - 1.0).max() < 1e-13
    # the row (1, 3): mean 2, biased variance 1 -> (-1, 1) / sqrt(1 + eps)
    two = oracle.layernorm_rows(np.array([[1.0, 3.0]]), np.array([2.0, 2.0]), np.array([0.5, -0.5]), 3.0)
    assert np.array_equal(two, np.array([[-1.0 / 2.0 * 2.0 + 0.5, 1.0 / 2.0 * 2.0 - 0.5]]))


def test_non_finite_rows_follow_torch_float64():
    """Rows holding +inf, -inf or NaN are outside the GPU's tested contract, but the oracle's branches for them (the
    NaN-propagating row maximum, logsumexp of an infinite maximum) are code like any other: pinned against torch's
    CPU float64 softmax and logsumexp, which take the same limits."""
    inf, nan = float("inf"), float("nan")
    rows = np.array([
        [1.0, 2.0, -inf, 0.5],       # a -inf entry: probability 0
        [-inf, -inf, -inf, -inf],    # all -inf: softmax NaN (0/0), logsumexp -inf
        [1.0, inf, 3.0, 2.0],        # a +inf entry: logsumexp +inf, softmax NaN at the inf (inf - inf)
        [1.0, nan, 3.0, 2.0],        # NaN anywhere poisons the row
        [nan, 1.0, 2.0, 3.0],        # ... also in the first place
        [0.0, 1.0, 2.0, 3.0],
    ])
    t = torch.from_numpy(rows)
    # (each row enters as the bias of a zero product: through a matrix product an infinity times zero would be NaN already)
    x0, w0 = np.zeros((1, 1)), np.zeros((4, 1))
    sm = np.concatenate([oracle.fused_linear_epilogue(x0, w0, r.copy(), [("bias",), ("softmax",)]) for r in rows])
    ref = torch.softmax(t, dim=-1).numpy()
    assert np.array_equal(np.isnan(sm), np.isnan(ref))
    assert np.allclose(sm[~np.isnan(ref)], ref[~np.isnan(ref)], rtol=1e-15, atol=0)
    lse = np.concatenate([oracle.fused_linear_epilogue(x0, w0, r.copy(), [("bias",), ("logsumexp",)]).reshape(-1) for r in rows])
    ref = torch.logsumexp(t, dim=-1).numpy()
    assert np.array_equal(np.isnan(lse), np.isnan(ref)), (lse, ref)
    fin = ~np.isnan(ref)
    assert np.array_equal(np.isinf(lse[fin]), np.isinf(ref[fin])) and np.array_equal(np.sign(lse[fin & np.isinf(ref)]), np.sign(ref[fin & np.isinf(ref)]))
    assert np.allclose(lse[fin & np.isfinite(ref)], ref[fin & np.isfinite(ref)], rtol=1e-15, atol=0)
