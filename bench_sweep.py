#!/usr/bin/env python3
"""Throughput surface of the self-join kernel over data set size and dimensionality.

The counterpart of the paper's Synth experiment (Section 4.2: uniformly distributed points,
|D| = 10^(3 + i/3), d = 64 .. 4096, kernel throughput only).  Points are U[0,1) rounded to FP16,
drawn on the device from a fixed seed; epsilon = 0, so only the n self pairs are written and the
time is that of norms + Gram + threshold.  Prints one JSON line per (n, d) and, with --table, a
markdown table of the derived throughput 2 n^2 d / t (the paper's convention) and of the executed
matrix-core throughput (upper-triangular tiles only) of the join kernel.

    python bench_sweep.py [--table] [--max-n 1000000] [--dims 64,128,...]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dims", default="64,128,256,512,1024,2048,4096")
    ap.add_argument("--min-exp", type=int, default=0, help="first i of n = 10^(3 + i/3)")
    ap.add_argument("--max-n", type=int, default=1_000_000)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--table", action="store_true")
    args = ap.parse_args()

    import torch

    import paper_2508_21230_amd as pkg

    dims = [int(x) for x in args.dims.split(",")]
    sizes = []
    i = args.min_exp
    while round(10 ** (3 + i / 3)) <= args.max_n:
        sizes.append(int(round(10 ** (3 + i / 3))))
        i += 1
    ej = pkg.EJoin(0)
    ej.reserve(max(sizes), max(dims))
    rows = {}
    for d in dims:
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(7000 + d)
        nmax = max(sizes)
        X = torch.empty((nmax, d), dtype=torch.float16, device="cuda:0")
        step_rows = max(1, (1 << 28) // d)
        for r0 in range(0, nmax, step_rows):  # in pieces: the FP32 draw of the whole set would not be needed at once
            r1 = min(nmax, r0 + step_rows)
            X[r0:r1] = torch.rand((r1 - r0, d), generator=gen, device="cuda:0", dtype=torch.float32).to(torch.float16)
        for n in sizes:
            Xd = X[:n].view(torch.int16)
            cap = n + 4096
            pairs = torch.empty((cap, 2), dtype=torch.int32, device="cuda:0")
            npairs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
            step = lambda: ej.selfjoin_pairs(Xd, 0.0, cap, pairs=pairs, dist2=None, n_pairs=npairs, with_dist2=False)
            step()
            torch.cuda.synchronize()
            ej.set_profiling(True)
            prep, join = [], []
            for _ in range(args.reps):
                step()
                a, b = ej.last_kernel_ms()
                prep.append(a)
                join.append(b)
            ej.set_profiling(False)
            jm, pm = min(join), min(prep)
            tiles = pkg.tiles_evaluated(n)
            rec = {"n": n, "d": d, "join_ms": jm, "prep_ms": pm, "pairs_found": int(npairs.cpu()[0]),
                   "derived_tflops": 2.0 * n * n * d / ((jm + pm) * 1e-3) / 1e12,
                   "executed_tflops": 2.0 * 256 * 256 * d * tiles / (jm * 1e-3) / 1e12}
            rows[(n, d)] = rec
            print(json.dumps(rec), flush=True)
            del pairs
        del X
    if args.table:
        for key, title in (("derived_tflops", "derived TFLOP/s, 2 n^2 d / (preparation + join kernel time)"),
                           ("executed_tflops", "executed matrix-core TFLOP/s of the join kernel")):
            print(f"\n{title}\n")
            print("| n \\ d | " + " | ".join(str(d) for d in dims) + " |")
            print("|---|" + "---|" * len(dims))
            for n in sizes:
                print(f"| {n} | " + " | ".join(f"{rows[(n, d)][key]:.0f}" for d in dims) + " |")


if __name__ == "__main__":
    main()
