"""GPU parity of the persistent perceptron chain (every layer of a batch-1 perceptron in one launch)
against the CPU oracle's chain of fused linear calls in float64."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_16964_amd import binding, inputs

from parity import assert_close

pytestmark = pytest.mark.gpu

F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16
DEV = "cuda:0"


def announce(*a):
    print("[case]", *a, flush=True)


def chain_factor(dtype, layers):
    """Allowance of a chain relative to one fused call's.  2-byte dtypes: every layer boundary rounds the activations
    to the storage dtype (as separate calls would), L independent roundings of the same relative size that pass
    through the remaining layers with a gain of about one and add in quadrature: sqrt(L).  fp32: the activations are
    not rounded again, so a chain gets the single call's 1e-4."""
    return 1.0 if dtype == torch.float32 else float(layers) ** 0.5


def random_chain(seed, widths, dtype, acts, bias=True):
    rng = np.random.default_rng(seed)
    x = torch.from_numpy(rng.standard_normal(widths[0]).astype(np.float32)).to(dtype)
    ws, bs = [], []
    for k, n in zip(widths, widths[1:]):
        a = np.sqrt(6.0 / k)
        ws.append(torch.from_numpy(rng.uniform(-a, a, (n, k)).astype(np.float32)).to(dtype))
        bs.append(torch.from_numpy(rng.uniform(-0.1, 0.1, n).astype(np.float32)).to(dtype) if bias else None)
    return x, ws, bs, list(acts)


def oracle_chain(x, ws, bs, acts):
    h = inputs.to_f64(x).reshape(1, -1)
    for w, b, act in zip(ws, bs, acts):
        ep = ([("bias",)] if b is not None else []) + ([(act,)] if act else [])
        h = oracle.fused_linear_epilogue(h, inputs.to_f64(w), inputs.to_f64(b), ep)
    return h.reshape(-1)


def run_chain(x, ws, bs, acts):
    d = lambda t: None if t is None else t.to(DEV)
    out = binding.mlp_chain(d(x), [d(w) for w in ws], [d(b) for b in bs], acts)
    torch.cuda.synchronize()
    return out.cpu()


@pytest.mark.parametrize("dtype,widths,acts,bias", [
    (F32, [64, 64], ["relu"], True),                                       # one layer: no barrier at all
    (F32, [256, 512, 128, 16], ["relu", "relu", None], True),              # fewer rows than one per wave on the chip
    (F32, [1024, 4096, 4096, 1000], ["relu", "gelu_tanh", None], True),    # ragged last layer
    (BF16, [512, 2048, 2048, 512], ["gelu_erf", "relu", "relu"], False),
    (F16, [2048, 8200, 264], ["relu", None], True),                        # more row blocks than workgroups
    (F32, [4, 20, 4], ["relu", "relu"], True),                             # tiny: a K of one 16-byte chunk
    (BF16, [4096] * 5, ["relu"] * 4, True),
    (F32, [20000, 96, 20000, 8], ["relu", "relu", None], True),            # long input vectors, layers with few rows
    (F16, [600, 16384, 600], ["gelu_tanh", None], True),
])
def test_chain_matches_oracle(dtype, widths, acts, bias):
    announce("chain", dtype, widths, acts, bias)
    x, ws, bs, acts = random_chain(len(widths) * 7 + widths[0], widths, dtype, acts, bias)
    got = run_chain(x, ws, bs, acts)
    assert_close(got, oracle_chain(x, ws, bs, acts), dtype, factor=chain_factor(dtype, len(ws)))


@pytest.mark.parametrize("wdtype,widths,acts", [
    (BF16, [4096, 4096, 4096, 4096], ["relu", "relu", "relu"]),
    (F16, [1024, 2048, 1000], ["gelu_tanh", None]),
    (BF16, [8, 24, 8], ["relu", None]),                                    # a W row of one 16-byte chunk
    (BF16, [20000, 96, 4104], ["relu", "relu"]),
])
def test_chain_with_reduced_precision_weights(wdtype, widths, acts):
    """fp32 input, biases, activations and output; weights stored in bf16 / fp16.  The oracle gets the same stored
    weights (upcast exactly), so the comparison is at the fp32 tolerance: the precision was reduced when the
    weights were prepared, not by the kernel."""
    announce("chain mixed", wdtype, widths, acts)
    x, ws, bs, acts = random_chain(31 + len(widths), widths, F32, acts)
    ws = [w.to(wdtype) for w in ws]
    got = run_chain(x, ws, bs, acts)
    assert got.dtype == F32
    assert_close(got, oracle_chain(x, ws, bs, acts), F32)


def test_chain_equals_the_separate_calls_bit_for_bit_in_fp32():
    """fp32: a layer in the chain and the same layer as its own fused call sum in different orders, so only the
    oracle decides; but two runs of the chain must agree exactly (fixed summation order, no atomics)."""
    announce("chain reproducible")
    x, ws, bs, acts = random_chain(5, [4096, 4096, 4096], F32, ["relu", "relu"])
    a = run_chain(x, ws, bs, acts)
    b = run_chain(x, ws, bs, acts)
    assert torch.equal(a, b)


def test_chain_back_to_back_calls_leave_the_barrier_state_clean():
    """200 calls queued without a host synchronisation in between, on one workspace: every call finds the barrier
    words at zero (the last workgroup of a call resets them), no wait runs out, and the result never changes."""
    announce("chain back to back")
    x, ws, bs, acts = random_chain(9, [2048, 4096, 4096, 2048], BF16, ["relu", "gelu_tanh", None])
    d = lambda t: t.to(DEV)
    call = binding.ChainCall(d(x), [d(w) for w in ws], [d(b) for b in bs], acts)
    first = call.run().clone()
    for _ in range(200):
        call.run()
    torch.cuda.synchronize()
    assert not call.barrier_error()
    assert (call.workspace[:2560] == 0).all()
    assert torch.equal(call.out, first)
    assert_close(call.out.cpu(), oracle_chain(x, ws, bs, acts), BF16, factor=chain_factor(BF16, len(ws)))


def test_m1_chain_in_one_launch():
    """bench.py's workload m2: the batch-1 perceptron of m1 (8 layers of 4096 x 4096, fp32) in one launch."""
    ch = inputs.make_chain()
    announce("m2", len(ch.ws))
    acts = ["relu"] * len(ch.ws)
    got = run_chain(ch.x, ch.ws, ch.bs, acts)
    assert_close(got.reshape(-1), oracle_chain(ch.x, ch.ws, ch.bs, acts), F32, "m2 end to end")


def test_chain_rejects_what_it_cannot_run():
    d = lambda t: t.to(DEV)
    x, ws, bs, acts = random_chain(1, [64, 32, 16], F32, ["relu", None])
    with pytest.raises(binding.FleError):
        binding.mlp_chain(d(x), [d(ws[0]), d(ws[0])], [None, None], acts)       # layer 1 takes 64 inputs, layer 0 gives 32
    x, ws, bs, acts = random_chain(1, [6, 8], F32, ["relu"])
    with pytest.raises(binding.FleError):
        binding.mlp_chain(d(x), [d(w) for w in ws], [None], acts)                # k = 6 floats is not a multiple of 16 bytes
    with pytest.raises(KeyError):
        binding.mlp_chain(d(x), [d(w) for w in ws], [None], ["softmax"])


def test_chain_in_a_hip_graph():
    """One ordinary kernel launch, no memset, no allocation: the chain can be captured and replayed; every replay
    reproduces the eager result bit for bit on changed inputs and leaves the barrier state clean."""
    announce("chain in a graph")
    x, ws, bs, acts = random_chain(12, [1024, 2048, 2048, 512], F32, ["relu", "relu", None])
    d = lambda t: t.to(DEV)
    xg = d(x)
    call = binding.ChainCall(xg, [d(w) for w in ws], [d(b) for b in bs], acts)
    call.run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        call.run()
    gen = torch.Generator().manual_seed(8)
    for rep in range(3):
        xg.copy_(torch.randn(xg.shape, generator=gen))
        eager = call.run().clone()
        torch.cuda.synchronize()
        call.out.fill_(-5.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(call.out, eager), "replay %d differs" % rep
    assert not call.barrier_error() and (call.workspace[:2560] == 0).all()
    assert_close(call.out.cpu(), oracle_chain(xg.cpu(), ws, bs, acts), F32)


def test_chain_that_gives_up_a_wait_poisons_its_result_and_says_so():
    """The give-up path, forced from the host: the error word is set before the call, so every wait ends at its first
    poll.  The kernel still terminates normally; the workgroups that gave up fill their share of out with NaN, the
    error word stays, the counters are back at zero, and the checked call raises.  After zeroing the state the same
    workspace gives the right result again."""
    announce("chain give-up")
    x, ws, bs, acts = random_chain(13, [1024, 4096, 4096, 1024], BF16, ["relu", "relu", None])
    d = lambda t: t.to(DEV)
    call = binding.ChainCall(d(x), [d(w) for w in ws], [d(b) for b in bs], acts)
    good = call.run_checked().clone()
    call.workspace[256:260].view(torch.int32).fill_(1)
    with pytest.raises(RuntimeError):
        call.run_checked()
    assert torch.isnan(call.out.float()).any()
    assert (call.workspace[:2560] == 0).all()                       # run_checked zeroed the state for the next call
    assert torch.equal(call.run_checked(), good)
    # the raw entry point: the error word survives the call, every counter is back at zero
    call.workspace[256:260].view(torch.int32).fill_(1)
    call.run()
    torch.cuda.synchronize()
    state = call.workspace[:2560].view(torch.int32).cpu()
    assert int(state[64]) == 1 and int(state.abs().sum()) == 1
