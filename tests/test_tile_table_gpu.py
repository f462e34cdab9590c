"""The per-call plan choice and the tuned-plan table on the GPU: every plan the table can name gives the oracle's
result, and a Call with a table runs the plan the table holds."""
import pytest
import torch

from paper_2511_16964_amd import binding, inputs

from parity import assert_close, oracle_rows, run_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant,split", [("tiled256", 1), ("tiled256", 4), ("tiled128", 1), ("tiled128", 8), ("skinny256", 0), ("general", 0)])
@pytest.mark.parametrize("row", [False, True])
def test_every_choice_matches_the_oracle(variant, split, row):
    dt = torch.bfloat16
    prob = inputs.random_problem(41, 200, 768, 1024, dt, ["bias", "gelu_tanh"] + (["layernorm"] if row else ["residual"]))
    got, call = run_gpu(prob, variant, poison=True, split=split)
    assert_close(got, oracle_rows(prob), dt, what="%s split %d: %s" % (variant, split, call.plan()))


def test_call_with_a_table_runs_the_tables_plan():
    dt = torch.bfloat16
    M, N, K = 256, 1024, 2048
    prob = inputs.random_problem(43, M, N, K, dt, ["bias", "relu"])
    ref = oracle_rows(prob)
    base = run_gpu(prob)[1].plan()
    t = binding.TileTable()
    t.entries[t.key(binding.BF16, M, N, K, prob.epilogue)] = {"variant": "tiled128", "split": 4}
    got, call = run_gpu(prob, poison=True, table=t)
    plan = call.plan()
    assert "tile=128x128" in plan and "split_k=4" in plan and plan != base
    assert_close(got, ref, dt, what="table plan")
    soft = inputs.random_problem(43, M, N, K, dt, ["bias", "softmax"])          # no entry for this class: the cost model decides
    got, call = run_gpu(soft, poison=True, table=t)
    assert "split_k=4" not in call.plan()
    assert_close(got, oracle_rows(soft), dt, what="no entry")
    got, call = run_gpu(prob, "tiled256", poison=True, table=t, split=1)       # an explicit choice wins over the table
    assert "tile=256x256" in call.plan()
    assert_close(got, ref, dt, what="explicit choice")
    shipped = binding.TileTable.load()                                          # every plan of the table in the package runs its shape
    for key, e in sorted(shipped.entries.items())[:12]:
        m, n, k = e["shape"]
        if m * n * k > 1 << 32:
            continue
        row = key.split(":")[1] == "1"
        p = inputs.random_problem(47, m, n, k, dt, ["bias", "layernorm"] if row else ["bias", "relu"])
        got, call = run_gpu(p, poison=True, table=shipped)
        rows = list(range(0, m, max(1, m // 8)))[:8]
        assert_close(got[rows], oracle_rows(p, rows), dt, what="shipped entry %s: %s" % (key, call.plan()))
