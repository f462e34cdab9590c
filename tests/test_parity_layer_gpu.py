"""GPU parity of one pre-norm transformer layer run as five fused calls (projection, attention, output
projection + residual + store + LayerNorm, perceptron up + GELU, perceptron down + residual + store +
LayerNorm) against the oracle's float64 layer.  Six values are stored in the storage dtype one after the
other on the way to a result (qkv, o, h, m, u, the result), each an independent relative rounding, so the
allowance is sqrt(6) times that of one fused call."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_16964_amd import binding, inputs
from parity import assert_close, to_dev

pytestmark = pytest.mark.gpu
LAYER_FACTOR = 6.0 ** 0.5
f64 = inputs.to_f64


def run_layer(lp):
    a = lp.attn
    d = to_dev
    call = binding.TransformerLayerCall(d(a.x), d(lp.n), d(a.w_qkv), d(a.b_qkv), d(a.w_o), d(a.b_o), a.heads, a.causal,
                                        (d(lp.g_mid), d(lp.be_mid), lp.eps), d(lp.w1), d(lp.b1), d(lp.w2), d(lp.b2), (d(lp.g_out), d(lp.be_out), lp.eps))
    x_out, n_out = call.run()
    torch.cuda.synchronize()
    return x_out.cpu(), n_out.cpu(), call


def oracle_layer(lp, seqs=None, tokens=None):
    a = lp.attn
    x, n = a.x, lp.n
    if seqs is not None:
        x, n = x[:seqs, :tokens], n[:seqs, :tokens]
    return oracle.transformer_layer(f64(x), f64(n), f64(a.w_qkv), f64(a.b_qkv), f64(a.w_o), f64(a.b_o), a.heads, a.causal,
                                    (f64(lp.g_mid), f64(lp.be_mid), lp.eps), f64(lp.w1), f64(lp.b1), f64(lp.w2), f64(lp.b2), (f64(lp.g_out), f64(lp.be_out), lp.eps))


@pytest.mark.parametrize("dtype,B,T,C,heads,Fh,causal", [
    (torch.bfloat16, 2, 150, 256, 4, 512, True),       # head dimension 64, ragged token count
    (torch.float16, 3, 77, 256, 2, 1024, False),       # head dimension 128, no mask
    (torch.bfloat16, 1, 300, 384, 12, 1000, True),     # head dimension 32, a perceptron width that is no multiple of 128
    (torch.bfloat16, 4, 1, 128, 4, 256, True),         # one token per sequence
])
def test_layer_matches_the_oracle(dtype, B, T, C, heads, Fh, causal):
    lp = inputs.make_layer("a1", seed=B + T, F=Fh, B=B, T=T, C=C, heads=heads, causal=causal, dtype=dtype)
    print("[case] layer", dtype, B, T, C, heads, Fh, causal, flush=True)
    x_out, n_out, call = run_layer(lp)
    rx, rn = oracle_layer(lp)
    assert_close(x_out.reshape(B * T, C), rx.reshape(B * T, C), dtype, "x'", factor=LAYER_FACTOR)
    assert_close(n_out.reshape(B * T, C), rn.reshape(B * T, C), dtype, "n'", factor=LAYER_FACTOR)
    # the intermediates the calls hand over, against the oracle's own values of them
    h_ref = oracle.attention_block(f64(lp.n), f64(lp.attn.w_qkv), f64(lp.attn.b_qkv), f64(lp.attn.w_o), f64(lp.attn.b_o), heads, causal, residual=f64(lp.attn.x))
    assert_close(call.h.cpu(), h_ref.reshape(B * T, C), dtype, "h (store)", factor=3.0 ** 0.5)


def test_layer_at_the_benchmark_size_on_the_first_tokens():
    """The benchmark's shape and launch configuration: under the causal mask the first tokens of a sequence
    depend on nothing after them, so the oracle computes just those; plus a property of the whole output:
    undoing the last LayerNorm's affine step leaves rows of mean 0 and variance 1."""
    lp = inputs.make_layer("a1")
    B, T, C = lp.attn.x.shape
    print("[case] layer at full size", B, T, C, flush=True)
    x_out, n_out, _ = run_layer(lp)
    n_tok = 131
    rx, rn = oracle_layer(lp, 1, n_tok)
    assert_close(x_out[0, :n_tok], rx[0], torch.bfloat16, "x'", factor=LAYER_FACTOR)
    assert_close(n_out[0, :n_tok], rn[0], torch.bfloat16, "n'", factor=LAYER_FACTOR)
    assert torch.isfinite(x_out.float()).all()
    z = (n_out.reshape(B * T, C).double() - lp.be_out.double()) / lp.g_out.double()
    assert z.mean(dim=1).abs().max() < 2e-2
    assert (z.var(dim=1, unbiased=False) - 1).abs().max() < 5e-2
