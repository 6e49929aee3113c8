#!/usr/bin/env python3
"""Leave-one-out ablation of the join kernel's design elements (the counterpart of the paper's
Table "leave-one-out", Section 4.3, for this kernel's own optimisations).

Each variant is the same source built with one element taken out (paper_2508_21230_amd/build.py:
ABLATIONS; build them first with `python -m paper_2508_21230_amd.build --ablations`); all variants
compute the same pairs, which this script checks by comparing the number of pairs found.  "no
symmetry" runs the full library's two-set join of the data with itself (every tile of the square).
Prints one JSON line per (variant, workload) and a markdown table.

    python bench_ablation.py [--workloads 3,4,5] [--steps 2]
    python bench_ablation.py --variant no_swizzle --workloads 3 --n 400000 --steps 1     (one variant: counter runs under rocprofv3)
    python bench_ablation.py --experiments [--workloads 3,4,5]

--experiments runs the timing-only builds (results meaningless, see the top of csrc/ejoin.hip):
  hot_panels   every copy hits in the L2; join time and shader clock beside the full kernel's on the same data --
               what the memory-side fetch of the operand panels costs in clock on real operands;
  no_copies    no global->LDS copies after the first four slices: MFMAs, LDS reads and barriers as they are,
               on the operand bits those slices left in the LDS -- what feeding the LDS costs altogether;
  cycle_marks  s_memtime marks between the sections of a tile -- where a tile's time goes, per kind of wavefront.
Each variant also passes the parity rule against the CPU oracle on small cases (tests/test_gpu_ablations.py).
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
    ap.add_argument("--variant", default=None, help="run this variant only ('full', 'no_symmetry' or a name of build.ABLATIONS)")
    ap.add_argument("--experiments", action="store_true", help="run the timing-only builds hot_panels, no_copies and cycle_marks instead")
    args = ap.parse_args()
    if args.experiments:
        return experiments(args)

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
    if args.variant:
        variants = [v for v in variants if v[0] == args.variant]
        if not variants:
            sys.exit(f"unknown variant {args.variant}")
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
                if ref_found is not None:
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
    if args.variant:
        return
    print("\n| variant | " + " | ".join(f"w{w}: ms | TFLOP/s (2n²d/t) | vs full" for w in workloads) + " |")
    print("|---|" + "---|---|---|" * len(workloads))
    for name, _ in variants:
        cells = []
        for w in workloads:
            r, f = table[(name, w)], table[("full", w)]
            cells.append(f"{r['ms']:.1f} | {r['derived_tflops']:.0f} | {r['derived_tflops'] / f['derived_tflops']:.2f}")
        print(f"| {name} | " + " | ".join(cells) + " |")


def sclk_mhz():
    import glob
    import re
    for p in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        m = re.search(r"(\d+)\s*Mhz\s*\*", open(p).read())
        if m:
            return int(m.group(1))
    return 0


def experiments(args):
    import time

    import numpy as np
    import torch

    import datagen
    import paper_2508_21230_amd as pkg
    from paper_2508_21230_amd import build

    with open(os.path.join(ROOT, "paper_2508_21230_amd", "workloads_eps.json")) as f:
        eps_all = json.load(f)
    sections = ["tile cursor", "first slice", "middle slices", "last slice", "augmentation MFMAs + filter + exact path",
                "first fragments of the next tile (the mark waits for them: their latency)", "periodic re-alignment of the XCD's workgroups",
                "wait for the copies in flight before a re-alignment"]
    for w in [int(x) for x in args.workloads.split(",")]:
        spec = datagen.WORKLOADS[w]
        n, d, S = args.n or spec["n"], spec["d"], spec["selectivity"][0]
        eps = float(eps_all[str(w)]["eps"][str(S)]["eps"])
        Xd = torch.from_numpy(datagen.generate(w, n=n).view(np.int16)).to("cuda:0")
        cap = int(n * (S / 2 + 1) * 1.6 * (n / spec["n"])) + (1 << 20)
        pairs = torch.empty((cap, 2), dtype=torch.int32, device="cuda:0")
        d2 = torch.empty(cap, dtype=torch.float32, device="cuda:0")
        npairs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        tiles = pkg.tiles_evaluated(n)
        flop = 2.0 * 65536 * ((d + 63) // 64 * 64) * tiles
        # (no_copies computes every tile on the first tile's operands: compared output-free, epsilon = 0, so that the
        # rare path sees no more than the duplicates in either build)
        for name in ("full", "hot_panels", "full eps=0", "no_copies", "full", "hot_panels", "full eps=0", "no_copies"):
            ej = pkg.EJoin(0, lib_path=None if name.startswith("full") else os.path.join(build.ABLATION_DIR, f"libejoin_{name}.so"))
            eps_run = 0.0 if name in ("full eps=0", "no_copies") else eps
            step = lambda: ej.selfjoin_pairs(Xd, eps_run, cap, pairs=pairs, dist2=d2, n_pairs=npairs)
            step()
            torch.cuda.synchronize()
            ej.set_profiling(True)
            ms, clk = [], []
            for _ in range(args.steps):
                step()
                time.sleep(0.4 * 1e-3 * max(ms[-1] if ms else 100.0, 10.0))  # sample the clock while the kernel runs
                clk.append(sclk_mhz())
                ms.append(ej.last_kernel_ms()[1])
            ej.set_profiling(False)
            t = sum(ms) / len(ms)
            print(json.dumps({"experiment": name, "workload": w, "n": n, "d": d, "join_ms": t, "executed_tflops": flop / t / 1e9,
                              "frac_of_peak": flop / t / 1e9 / 2500.0, "sclk_MHz": sum(clk) / len(clk)}), flush=True)
            ej.close()
        ej = pkg.EJoin(0, lib_path=os.path.join(build.ABLATION_DIR, "libejoin_cycle_marks.so"))
        ej.selfjoin_pairs(Xd, eps, cap, pairs=pairs, dist2=d2, n_pairs=npairs)
        torch.cuda.synchronize()
        marks = pairs.view(torch.int64).flatten()[cap - 16:cap]
        marks.zero_()
        ej.set_profiling(True)
        ej.selfjoin_pairs(Xd, eps, cap, pairs=pairs, dist2=d2, n_pairs=npairs)
        ms = ej.last_kernel_ms()[1]
        torch.cuda.synchronize()
        v = marks.cpu().numpy().astype(float) / (4.0 * tiles)  # 4 wavefronts of each kind per workgroup, tiles / 256 tiles per workgroup, 256 workgroups
        rec = {"experiment": "cycle_marks", "workload": w, "n": n, "d": d, "join_ms": ms, "unit": "s_memtime ticks per tile and wavefront",
               "waves_0_3_no_copies": {sections[k]: round(v[k], 1) for k in range(8)}, "waves_4_7_copying": {sections[k]: round(v[8 + k], 1) for k in range(8)},
               "ticks_per_tile": round(v[:8].sum(), 1), "mfma_ticks_if_busy": "1024 cycles per slice and SIMD, 512 for the augmentation step"}
        print(json.dumps(rec), flush=True)
        ej.close()
        del pairs, d2, Xd


if __name__ == "__main__":
    main()
