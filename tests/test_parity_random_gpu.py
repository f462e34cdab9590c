"""GPU parity on seeded random problems: random shapes (ragged, tiny, thin, wide), dtypes, epilogue chains,
leading dimensions and kernel variants, each compared element by element with the CPU oracle.  The fixed
cases elsewhere pin the known tile boundaries; this sweep looks for the combinations nobody thought of."""
import numpy as np
import pytest
import torch

from paper_2511_16964_amd import binding, inputs

from parity import BLOCK_FACTOR, assert_close, attention_reference, oracle_grouped, oracle_rows, run_grouped_gpu

pytestmark = pytest.mark.gpu

DTYPES = [torch.float32, torch.bfloat16, torch.float16]
OPS = ["bias", "scale", "relu", "gelu_erf", "gelu_tanh", "residual"]
ROW_OPS = ["layernorm", "softmax", "logsumexp"]


def random_chain(rng):
    pre = [OPS[i] for i in rng.integers(0, len(OPS), rng.integers(0, 4))]
    chain = list(pre)
    if rng.random() < 0.5:
        row = ROW_OPS[rng.integers(0, 3)]
        chain.append(row)
        if row != "logsumexp":
            chain += [OPS[i] for i in rng.integers(0, len(OPS), rng.integers(0, 3))]
    return chain


def random_dims(rng):
    kind = rng.integers(0, 7)
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
    if kind == 5:      # perceptron layers
        return int(rng.integers(1, 33)), int(rng.integers(8, 64)) * 128, int(rng.integers(4, 20)) * 256
    return int(rng.integers(200, 1000)), int(rng.integers(200, 2000)), int(rng.integers(8, 128)) * 8   # several large tiles


@pytest.mark.parametrize("seed", range(160))
def test_random_problem_matches_oracle(seed):
    rng = np.random.default_rng(10_000 + seed)
    dtype = DTYPES[rng.integers(0, 3)]
    M, N, K = random_dims(rng)
    chain = random_chain(rng)
    prob = inputs.random_problem(20_000 + seed, M, N, K, dtype, chain)
    dev = "cuda:0"
    # operands inside larger buffers: leading dimensions larger than the row, optionally misaligned starts
    def place(t, pad_cols, shift):
        if t is None:
            return None
        if t.dim() == 1:
            buf = torch.zeros(t.numel() + shift, dtype=t.dtype, device=dev)
            buf[shift:] = t.to(dev)
            return buf[shift:]
        buf = torch.zeros(t.shape[0], t.shape[1] + pad_cols + shift, dtype=t.dtype, device=dev)
        view = buf[:, shift:shift + t.shape[1]]
        view.copy_(t.to(dev))
        return view
    pad = int(rng.integers(0, 3)) * 8
    shift = int(rng.integers(0, 2)) * int(rng.integers(0, 4)) if rng.random() < 0.3 else 0
    x, w, b = place(prob.x, pad, shift), place(prob.w, pad, shift), place(prob.b, 0, shift)
    ep = []
    for e in prob.epilogue:
        if e[0] == "residual":
            ep.append(("residual", place(e[1], pad, shift)))
        elif e[0] == "layernorm":
            ep.append(("layernorm", place(e[1], 0, shift), place(e[2], 0, shift), e[3]))
        else:
            ep.append(e)
    variants = ["auto", "auto", "general"]
    if K % 8 == 0 and shift == 0:
        variants += ["tiled", "tiled128", "tiled256"]
        if M <= 32:
            variants.append("thin")
        if M <= 256 and K % 64 == 0 and N % 4 == 0:
            variants += ["skinny", "skinny256"]
            if dtype != torch.float32 and K % 256 == 0:
                variants.append("skinnyseq")
    variant = variants[rng.integers(0, len(variants))]
    print("[case] seed %d %s M=%d N=%d K=%d %s pad=%d shift=%d %s" % (seed, str(dtype)[6:], M, N, K, variant, pad, shift, chain), flush=True)
    try:
        call = binding.Call(x, w, b, ep, variant=variant)
    except binding.FleError as err:
        assert variant != "auto" and err.status == 5, err      # a forced variant may refuse; the automatic plan never does
        call = binding.Call(x, w, b, ep)
    out = call.run()
    torch.cuda.synchronize()
    assert_close(out.cpu(), oracle_rows(prob), dtype, "%s %s" % (chain, call.plan()))


@pytest.mark.parametrize("seed", range(40))
def test_random_grouped_problem_matches_oracle(seed):
    rng = np.random.default_rng(30_000 + seed)
    dtype = DTYPES[rng.integers(0, 3)]
    G = int(rng.integers(1, 90))
    total = int(rng.integers(1, 1500))
    counts = inputs.routed_counts(seed, total, G, skew=float(rng.choice([0.2, 1.0, 5.0])))
    N = int(rng.integers(1, 600))
    K = int(rng.integers(1, 30)) * 8
    chain = random_chain(rng)
    gp = inputs.random_grouped(40_000 + seed, counts, N, K, dtype, chain, shared_bias=bool(rng.integers(0, 2)))
    variant = ["auto", "tiled128", "tiled256"][rng.integers(0, 3)]
    print("[case] grouped seed %d %s G=%d rows=%d N=%d K=%d %s %s" % (seed, str(dtype)[6:], G, total, N, K, variant, chain), flush=True)
    got, call = run_grouped_gpu(gp, variant)
    assert_close(got, oracle_grouped(gp), dtype, "%s %s" % (chain, call.plan()))


@pytest.mark.parametrize("seed", range(80))
def test_random_attention_matches_oracle(seed):
    """Random sequence lengths (1 .. 700, mostly ragged against the 128-query and 64-key blocks), head counts,
    batch sizes, all four head dimensions and both dtypes, without mask, causal and causal over groups of tokens, default and explicit
    scales, q / k / v as views of one fused buffer or as separate tensors with padded token strides."""
    import oracle
    rng = np.random.default_rng(5000 + seed)
    dtype = [torch.bfloat16, torch.float16][rng.integers(0, 2)]
    D = [32, 64, 128, 256][rng.integers(0, 4)]
    T = int(rng.integers(1, 700)) if rng.random() < 0.8 else int(rng.integers(1, 6)) * 128
    B, H = int(rng.integers(1, 4)), int(rng.integers(1, 12))
    causal = [0, 1, int(rng.integers(2, 200))][rng.integers(0, 3)]   # none, per token, per group of tokens
    scale = None if rng.random() < 0.6 else float(rng.uniform(0.02, 0.5))
    spread = float(rng.choice([0.3, 1.0, 2.5]))
    print("[case] random attention", seed, dtype, D, T, B, H, causal, scale, spread, flush=True)
    qkv = inputs.make_qkv(seed, B, T, H, D, dtype, spread)
    dev = qkv.to("cuda:0")
    layout = rng.random()
    if layout < 0.4:
        q, k, v = dev[:, :, 0], dev[:, :, 1], dev[:, :, 2]
    elif layout < 0.6:   # sequence-first memory, viewed batch-first
        tb = dev.transpose(0, 1).contiguous()
        q, k, v = (tb[:, :, i].transpose(0, 1) for i in range(3))
    else:   # separate buffers, token stride padded by 8 .. 64 elements
        def padded(t):
            pad = int(rng.integers(1, 9)) * 8
            buf = torch.zeros(B * T, H * D + pad, device="cuda:0", dtype=dtype)
            buf[:, :H * D] = t.reshape(B * T, H * D)
            return buf[:, :H * D].view(B, T, H, D)
        q, k, v = padded(dev[:, :, 0]), padded(dev[:, :, 1]), padded(dev[:, :, 2])
    got = binding.attention(q, k, v, causal, scale)
    torch.cuda.synchronize()
    f = inputs.to_f64(qkv)
    ref, extra = attention_reference(f[:, :, 0], f[:, :, 1], f[:, :, 2], causal, dtype, scale)
    assert_close(got.cpu(), ref, dtype, "seed %d" % seed, extra=extra)


@pytest.mark.parametrize("seed", range(12))
def test_random_attention_block_matches_oracle(seed):
    import oracle
    rng = np.random.default_rng(7000 + seed)
    dtype = [torch.bfloat16, torch.float16][rng.integers(0, 2)]
    D = [64, 128][rng.integers(0, 2)]
    heads = int(rng.integers(1, 7))
    B, T = int(rng.integers(1, 4)), int(rng.integers(1, 400))
    causal, bias, residual = bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    print("[case] random attention block", seed, dtype, D, heads, B, T, causal, bias, residual, flush=True)
    ap = inputs.make_attention("a1", seed, B=B, T=T, C=heads * D, heads=heads, causal=causal, dtype=dtype, bias=bias, residual=residual)
    d = lambda t: None if t is None else t.to("cuda:0")
    x = d(ap.x)
    got = binding.attention_block(x, d(ap.w_qkv), d(ap.b_qkv), d(ap.w_o), d(ap.b_o), heads, causal, residual=x if residual else None)
    torch.cuda.synchronize()
    f = inputs.to_f64
    ref = oracle.attention_block(f(ap.x), f(ap.w_qkv), f(ap.b_qkv), f(ap.w_o), f(ap.b_o), heads, causal, residual=f(ap.residual))
    assert_close(got.cpu(), ref, dtype, "seed %d" % seed, factor=BLOCK_FACTOR)
