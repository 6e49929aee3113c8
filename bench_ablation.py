#!/usr/bin/env python3
"""Leave-one-out ablation of the join kernel's design elements (the counterpart of the paper's
Table "leave-one-out", Section 4.3, for this kernel's own optimisations).

Each variant is the same source built with one element taken out (paper_2508_21230_amd/build.py:
ABLATIONS; build them first with `python -m paper_2508_21230_amd.build --ablations`); all variants
compute the same pairs, which this script checks by comparing the number of pairs found.  "no
symmetry" runs the full library's two-set join of the data with itself (every tile of the square).
Prints one JSON line per (variant, workload) and a markdown table.

    python bench_ablation.py [--workloads 3,4,5] [--steps 2]
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
    ap.add_argument("--workloads", default="3,4,5")
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--n", type=int, default=None, help="override the number of points (quick runs)")
    args = ap.parse_args()

    import numpy as np
    import torch

    import datagen
    import paper_2508_21230_amd as pkg
    from paper_2508_21230_amd import build

    with open(os.path.join(ROOT, "paper_2508_21230_amd", "workloads_eps.json")) as f:
        eps_all = json.load(f)
    variants = [("full", None)]
    for name in build.ABLATIONS:
        path = os.path.join(build.ABLATION_DIR, f"libejoin_{name}.so")
        if not os.path.exists(path):
            sys.exit(f"{path} is missing: run `python -m paper_2508_21230_amd.build --ablations` first")
        variants.append((name, path))
    variants.append(("no_symmetry", None))
    table = {}
    workloads = [int(w) for w in args.workloads.split(",")]
    for w in workloads:
        spec = datagen.WORKLOADS[w]
        n, d, S = args.n or spec["n"], spec["d"], spec["selectivity"][0]
        eps = float(eps_all[str(w)]["eps"][str(S)]["eps"])
        Xd = torch.from_numpy(datagen.generate(w, n=n).view(np.int16)).to("cuda:0")
        cap = int(n * (S / 2 + 1) * 1.6 * (n / spec["n"])) + (1 << 20)
        pairs = torch.empty((2 * cap, 2), dtype=torch.int32, device="cuda:0")
        d2 = torch.empty(2 * cap, dtype=torch.float32, device="cuda:0")
        npairs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        ref_found = None
        for name, path in variants:
            ej = pkg.EJoin(0, lib_path=path)
            if name == "no_symmetry":
                step = lambda: ej.join_pairs(Xd, Xd, eps, 2 * cap, pairs=pairs, dist2=d2, n_pairs=npairs)
            else:
                step = lambda: ej.selfjoin_pairs(Xd, eps, 2 * cap, pairs=pairs, dist2=d2, n_pairs=npairs)
            step()
            torch.cuda.synchronize()
            ej.set_profiling(True)
            ms = []
            for _ in range(args.steps):
                step()
                a, b = ej.last_kernel_ms()
                ms.append(a + b)
            ej.set_profiling(False)
            found = int(npairs.cpu()[0])
            if name == "no_symmetry":
                # ordered pairs, self pairs included once: 2 * (found_self - n) + n, up to pairs on the threshold itself
                # (the matrix cores' sum of a step is not symmetric in its operands to the last bit, so (i, j) and
                # (j, i) of a pair whose distance is epsilon to FP32 resolution can fall on different sides)
                want = 2 * (ref_found - n) + n
                assert abs(found - want) <= 1e-6 * want, (found, ref_found)
            elif ref_found is None:
                ref_found = found
            else:
                assert found == ref_found, (name, found, ref_found)
            t = min(ms)
            rec = {"variant": name, "workload": w, "n": n, "d": d, "ms": t, "derived_tflops": 2.0 * n * n * d / (t * 1e-3) / 1e12,
                   "pairs_found": found}
            table[(name, w)] = rec
            print(json.dumps(rec), flush=True)
            ej.close()
        del pairs, d2, Xd
    print("\n| variant | " + " | ".join(f"w{w}: ms | TFLOP/s (2n²d/t) | vs full" for w in workloads) + " |")
    print("|---|" + "---|---|---|" * len(workloads))
    for name, _ in variants:
        cells = []
        for w in workloads:
            r, f = table[(name, w)], table[("full", w)]
            cells.append(f"{r['ms']:.1f} | {r['derived_tflops']:.0f} | {r['derived_tflops'] / f['derived_tflops']:.2f}")
        print(f"| {name} | " + " | ".join(cells) + " |")


if __name__ == "__main__":
    main()
