"""GPU parity of the store op: one call hands over both the values at a point of the epilogue chain
(say x + f(x), the stream a pre-norm transformer layer carries on) and what the rest of the chain
makes of them (say their LayerNorm, the next layer's input), the multi-output form of the fused
operator chains of section 3.1.  Each kernel family writes the copy in its own way (whole vectors,
single elements on edge tiles, the finalize pass), so every family is driven here."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_16964_amd import binding, inputs
from parity import TOL, assert_close, to_dev

pytestmark = pytest.mark.gpu

F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16


def run_both(prob, variant="auto", offsets=None, split=0):
    """(gpu out, gpu store targets, oracle out, oracle store targets) of one problem."""
    ep_dev = [tuple(to_dev(a) if isinstance(a, torch.Tensor) else a for a in e) for e in prob.epilogue]
    kw = {}
    if offsets is not None:
        kw["offsets"] = torch.tensor(offsets, dtype=torch.int64, device="cuda:0")
    if split:
        kw["split"] = split
    call = binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), ep_dev, variant=variant, **kw)
    out = call.run()
    torch.cuda.synchronize()
    ep64 = inputs.epilogue_f64(prob.epilogue)
    if offsets is None:
        ref = oracle.fused_linear_epilogue(inputs.to_f64(prob.x), inputs.to_f64(prob.w), inputs.to_f64(prob.b), ep64)
    else:
        ref = oracle.grouped_fused_linear_epilogue(inputs.to_f64(prob.x), inputs.to_f64(prob.w), inputs.to_f64(prob.b),
                                                   offsets, ep64)
    got_t = [e[1].cpu() for e in ep_dev if e[0] == "store"]
    ref_t = [e[1] for e in ep64 if e[0] == "store"]
    return out.cpu(), got_t, ref, ref_t, call


def check(prob, variant="auto", offsets=None, expect=None, split=0):
    out, got_t, ref, ref_t, call = run_both(prob, variant, offsets, split)
    if expect is not None:
        assert expect in call.plan(), call.plan()
    assert_close(out, ref, prob.dtype, "out")
    assert len(got_t) == len(ref_t) >= 1
    for i, (g, r) in enumerate(zip(got_t, ref_t)):
        assert not np.isnan(r).any()
        assert_close(g, r, prob.dtype, "store %d" % i)


PRE_NORM = ["bias", "residual", "store", "layernorm"]

CASES = [
    # (dtype, M, N, K, kinds, variant, expected family or None)
    (BF16, 300, 768, 512, PRE_NORM, "auto", None),
    (BF16, 1024, 1024, 1024, PRE_NORM, "tiled", None),
    (BF16, 777, 1000, 520, PRE_NORM, "tiled", None),               # ragged M and N: edge tiles store element by element
    (BF16, 515, 1001, 333, PRE_NORM, "general", None),             # odd N: the scalar kernel
    (F16, 640, 512, 1024, PRE_NORM, "tiled128", None),
    (F32, 200, 384, 256, PRE_NORM, "auto", None),
    (F32, 513, 262, 132, ["bias", "store", "gelu_erf"], "tiled", None),           # N % 4 != 0: edge tiles in fp32
    (BF16, 64, 4096, 4096, PRE_NORM, "skinny", None),
    (BF16, 96, 2048, 1024, ["bias", "relu", "store", "scale", "residual", "store", "softmax"], "skinny128", None),
    (F16, 33, 1024, 2048, ["store", "bias", "gelu_tanh"], "skinny256", None),
    (BF16, 8, 4096, 4096, PRE_NORM, "thin", None),
    (F16, 3, 1024, 1536, ["bias", "store", "logsumexp"], "thin", None),
    (F32, 5, 768, 512, ["bias", "residual", "store", "layernorm"], "thin", None),
    (BF16, 256, 512, 8192, PRE_NORM, "auto", "split_k="),          # a shape the planner splits along K: the reduction pass stores
    (BF16, 16, 4096, 4096, PRE_NORM, "auto", "skinny"),
    (BF16, 1, 1, 1, ["store"], "auto", None),
    (BF16, 130, 256, 0, ["bias", "store", "relu"], "auto", None),  # K = 0: the copy holds the bias
]


@pytest.mark.parametrize("dtype,M,N,K,kinds,variant,expect", CASES)
def test_store_matches_the_oracle(dtype, M, N, K, kinds, variant, expect):
    prob = inputs.random_problem(4100 + M + N, M, N, K, dtype, kinds)
    check(prob, variant, expect=expect)


@pytest.mark.parametrize("dtype,M,N,K,variant,split", [
    (BF16, 128, 4096, 4096, "tiled", 0), (BF16, 300, 520, 576, "tiled", 3), (F32, 200, 262, 512, "tiled", 2),
    (F16, 16, 4096, 4096, "skinny", 0), (BF16, 40, 2048, 4096, "skinny", 4), (F32, 16, 4096, 8192, "skinny", 0),
])
def test_store_in_a_call_split_along_k(dtype, M, N, K, variant, split):
    """With K split, the pass that sums the slabs applies the ops and writes the copy."""
    prob = inputs.random_problem(5200 + M + N, M, N, K, dtype, ["bias", "gelu_tanh", "residual", "store", "scale", "layernorm"])
    out, got_t, ref, ref_t, call = run_both(prob, variant, None, split)
    assert "split_k=1 " not in call.plan(), call.plan()
    assert_close(out, ref, dtype, "out")
    assert_close(got_t[0], ref_t[0], dtype, "store")


def test_store_is_exact_on_integer_inputs():
    """Small-integer operands make the elementwise chain exact in every dtype: the copy must then
    equal the oracle's bit for bit, and untouched padding of a strided target keeps its fill."""
    M, N, K = 200, 320, 64
    prob = inputs.random_problem(77, M, N, K, BF16, ["bias", "relu", "scale", "residual", "store", "relu"], integer=True)
    wide = torch.full((M, N + 24), -3.0, dtype=BF16, device="cuda:0")
    ep_dev = []
    for e in prob.epilogue:
        if e[0] == "store":
            ep_dev.append(("store", wide[:, :N]))
        else:
            ep_dev.append(tuple(to_dev(a) if isinstance(a, torch.Tensor) else a for a in e))
    out = binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), ep_dev).run()
    torch.cuda.synchronize()
    ep64 = inputs.epilogue_f64(prob.epilogue)
    ref = oracle.fused_linear_epilogue(inputs.to_f64(prob.x), inputs.to_f64(prob.w), inputs.to_f64(prob.b), ep64)
    t_ref = [e[1] for e in ep64 if e[0] == "store"][0]
    assert np.array_equal(out.cpu().double().numpy(), ref)
    assert np.array_equal(wide[:, :N].cpu().double().numpy(), t_ref)
    assert bool((wide[:, N:] == -3.0).all())


@pytest.mark.parametrize("variant,N", [("auto", 512), ("tiled128", 512), ("tiled256", 512), ("auto", 513), ("auto", 518)])
def test_store_in_a_grouped_call(variant, N):
    counts = [0, 130, 1, 257, 64, 0, 31]
    gp = inputs.random_grouped(912, counts, N, 384, BF16, PRE_NORM)
    check(gp, variant, offsets=gp.offsets)


def test_store_in_a_thin_grouped_call():
    counts = [3, 0, 16, 7, 1, 12]
    gp = inputs.random_grouped(913, counts, 1024, 1024, BF16, ["bias", "store", "gelu_erf"])
    check(gp, "auto", offsets=gp.offsets)


def _random_dims(rng):
    kind = rng.integers(0, 6)
    if kind == 0:      # tiny
        return int(rng.integers(1, 40)), int(rng.integers(1, 70)), int(rng.integers(1, 70))
    if kind == 1:      # a few rows against a wide matrix (thin / skinny kernels)
        return int(rng.integers(1, 70)), int(rng.integers(1, 40)) * 64 + int(rng.integers(0, 2)) * int(rng.integers(1, 64)), int(rng.integers(1, 24)) * 64
    if kind == 2:      # tiled shapes with ragged edges
        return int(rng.integers(100, 700)), int(rng.integers(100, 900)), int(rng.integers(1, 40)) * 8
    if kind == 3:      # K that breaks the 16-byte rule
        return int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 300))
    if kind == 4:      # long K, few tiles (split K)
        return int(rng.integers(1, 200)), int(rng.integers(64, 400)), int(rng.integers(8, 40)) * 128
    return int(rng.integers(1, 33)), int(rng.integers(8, 64)) * 128, int(rng.integers(4, 20)) * 256   # perceptron layers


@pytest.mark.parametrize("seed", range(80))
def test_random_problem_with_stores_matches_oracle(seed):
    """Seeded random shapes, dtypes, chains, leading dimensions and variants, each chain with one or two
    stores before its row op; out and every store target are compared element by element."""
    rng = np.random.default_rng(30_000 + seed)
    dtype = [F32, BF16, F16][rng.integers(0, 3)]
    M, N, K = _random_dims(rng)
    elementwise = ["bias", "scale", "relu", "gelu_erf", "gelu_tanh", "residual"]
    chain = [elementwise[i] for i in rng.integers(0, 6, rng.integers(0, 4))]
    for _ in range(int(rng.integers(1, 3))):
        chain.insert(int(rng.integers(0, len(chain) + 1)), "store")
    if rng.random() < 0.6:
        row = ["layernorm", "softmax", "logsumexp"][rng.integers(0, 3)]
        chain.append(row)
        if row != "logsumexp":
            chain += [elementwise[i] for i in rng.integers(0, 6, rng.integers(0, 3))]
    prob = inputs.random_problem(31_000 + seed, M, N, K, dtype, chain)
    pad = int(rng.integers(0, 3)) * 8
    shift = int(rng.integers(1, 4)) if rng.random() < 0.15 else 0     # store targets that rule out vector stores

    def place(t):
        buf = torch.full((t.shape[0], t.shape[1] + pad + shift), -5.0, dtype=t.dtype, device="cuda:0")
        view = buf[:, shift:shift + t.shape[1]]
        view.copy_(t.to("cuda:0"))
        return view, buf
    ep, targets = [], []
    for e in prob.epilogue:
        if e[0] == "store":
            view, buf = place(e[1])
            targets.append((view, buf))
            ep.append(("store", view))
        else:
            ep.append(tuple(to_dev(a) if isinstance(a, torch.Tensor) else a for a in e))
    variants = ["auto", "auto", "general"]
    if K % 8 == 0:
        variants += ["tiled", "tiled128", "tiled256"]
        if M <= 32:
            variants.append("thin")
        if M <= 256 and K % 64 == 0 and N % 4 == 0:
            variants += ["skinny", "skinny256"]
    variant = variants[rng.integers(0, len(variants))]
    split = int(rng.integers(2, 5)) if (variant in ("tiled", "skinny") and K >= 512 and rng.random() < 0.5) else 0
    print("[case] seed %d %s M=%d N=%d K=%d %s split=%d pad=%d shift=%d %s" % (seed, str(dtype)[6:], M, N, K, variant, split, pad, shift, chain), flush=True)
    try:
        call = binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), ep, variant=variant, split=split)
    except binding.FleError as err:
        assert variant != "auto" and err.status == 5, err      # a forced variant may refuse; the automatic plan never does
        call = binding.Call(to_dev(prob.x), to_dev(prob.w), to_dev(prob.b), ep)
    out = call.run()
    torch.cuda.synchronize()
    ep64 = inputs.epilogue_f64(prob.epilogue)
    ref = oracle.fused_linear_epilogue(inputs.to_f64(prob.x), inputs.to_f64(prob.w), inputs.to_f64(prob.b), ep64)
    assert_close(out.cpu(), ref, dtype, "%s %s" % (chain, call.plan()))
    ref_t = [e[1] for e in ep64 if e[0] == "store"]
    assert len(ref_t) == len(targets)
    for i, ((view, buf), r) in enumerate(zip(targets, ref_t)):
        assert_close(view.cpu(), r, dtype, "store %d %s %s" % (i, chain, call.plan()))
        assert bool((buf[:, :shift] == -5.0).all()) and bool((buf[:, shift + N:] == -5.0).all()), "padding of store %d written" % i
