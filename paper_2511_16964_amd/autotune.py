"""Offline tuning of the plan (kernel family, tile, split of K): measures every candidate plan of a list of problem
classes on the GPU at hand through the C ABI's per-call plan choice and writes the fastest into a table that
``binding.Call(..., table=...)`` applies.  The paper credits autotuned tile choices for many of its best solutions
(Section 5.2, appendix on outlier tasks); here the table also shows how far the library's cost model is from the
measured optimum.

    python -m paper_2511_16964_amd.autotune [--out PATH] [--quick]
"""
from __future__ import annotations

import argparse
import sys
import time

import torch

from . import binding

CANDIDATES = [("auto", 0)] + [(v, s) for v in ("tiled256", "tiled128") for s in (1, 2, 4, 8, 16)] + \
    [("skinny", 0), ("skinny128", 0), ("skinny256", 0), ("skinnyseq", 0), ("thin", 0), ("general", 0)]


_flush = None


def time_call(call, iters=12):
    """Median time of one call in microseconds, each call timed on its own behind an overwrite of 768 MB that
    evicts L2 and the Infinity Cache: in a network a layer's weights are read once per pass, and a candidate that
    only wins because the same 100 - 250 MB of weights stay in the 256 MB cache from one timed call to the next (the
    tiled kernels against the streaming ones, up to 20 % in a back-to-back loop) would be the wrong choice there."""
    global _flush
    if _flush is None:
        _flush = torch.empty(768 << 20, dtype=torch.uint8, device="cuda:0")
    call.run()
    torch.cuda.synchronize()
    times = []
    for _ in range(iters):
        _flush.fill_(1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); call.run(); e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2] * 1e3


def tune(shapes, dtypes, log=print):
    dev = torch.device("cuda:0")
    table = binding.TileTable(meta={"device": torch.cuda.get_device_name(0), "made": time.strftime("%Y-%m-%d"),
                                    "unit": "microseconds per call, caches evicted before each", "library_version": binding.lib().fle_version()})
    for dt in dtypes:
        for (M, N, K) in shapes:
            x = torch.randn(M, K, device=dev).to(dt)
            w = (torch.rand(N, K, device=dev) * 2 - 1).mul_(K ** -0.5).to(dt)
            b = torch.zeros(N, device=dev, dtype=dt)
            g = torch.ones(N, device=dev, dtype=dt)
            for ep in ([("bias",), ("relu",)], [("bias",), ("layernorm", g, b, 1e-5)]):
                out = torch.empty(M, N, device=dev, dtype=dt)
                results = {}
                for variant, split in CANDIDATES:
                    if variant == "general" and M * N * K > (1 << 31):
                        continue
                    try:
                        call = binding.Call(x, w, b, ep, out=out, variant=variant, split=split)
                    except binding.FleError:
                        continue   # this plan cannot run the problem
                    results[(variant, split)] = time_call(call)
                auto = results[("auto", 0)]
                (bv, bs), bt = min(results.items(), key=lambda kv: kv[1])
                key = binding.TileTable.key(binding._dtype_code(dt), M, N, K, ep)
                if bt < 0.97 * auto:   # (within 3 % the cost model's own choice stands)
                    table.entries[key] = {"variant": bv, "split": bs, "us": round(bt, 2), "auto_us": round(auto, 2), "shape": [M, N, K]}
                log("%-9s %6d x %6d x %6d %-9s auto %9.1f us  best %-9s split %2d %9.1f us  (%.2fx)" % (
                    str(dt).replace("torch.", ""), M, N, K, "row op" if len(ep[1]) > 1 else "plain", auto, bv, bs, bt, auto / bt))
    return table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=binding.TileTable.DEFAULT_PATH)
    ap.add_argument("--quick", action="store_true", help="a handful of shapes only")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("autotune needs the GPU the table is for")
    Ms = [1, 16, 128, 4096] if args.quick else [1, 4, 16, 64, 256, 1024, 4096, 16384]
    NKs = [(4096, 4096)] if args.quick else [(1024, 1024), (4096, 4096), (4096, 16384), (16384, 4096), (32768, 8192)]
    shapes = [(M, N, K) for (N, K) in NKs for M in Ms]
    table = tune(shapes, [torch.bfloat16])
    table.save(args.out)
    print("wrote %d entries (plans that beat the cost model's choice by more than 3 %%) to %s" % (len(table.entries), args.out))


if __name__ == "__main__":
    main()
