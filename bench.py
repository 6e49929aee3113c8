#!/usr/bin/env python3
"""Benchmark of the epsilon self-join hot path on one MI355X.

One "step" = one pass of the whole hot path over one synthetic workload that is already resident
in HBM: norm kernel, counter reset, Gram + threshold + compaction kernel (pair list with dist2).
Prints ONE JSON line.  `value` is the paper's derived throughput 2*n^2*d / t (Section 4.1.1:
total operations of the all-pairs comparison divided by the measured time), which credits the
use of symmetry as speed; `roofline.achieved` counts only the matrix-core work actually
executed (upper-triangular 256x256 tiles) against the dense FP16 MFMA peak.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0  # MI355X dense FP16 MFMA, published

# Bytes k_join fetches into L2 from the memory side plus bytes it writes, per launch, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a copy of known size
# (profiles/k_join_workload3_hbm_counters.txt).  Only measured for the default workload.
MEASURED_TRAFFIC_BYTES = {(3, 16, "pairs"): 1.888e12}


def load_eps(workload: int, S: int) -> float:
    with open(os.path.join(ROOT, "paper_2508_21230_amd", "workloads_eps.json")) as f:
        return float(json.load(f)[str(workload)]["eps"][str(S)]["eps"])


def cpu_baseline(X, workload, eps, budget_rows):
    """The CPU oracle as it stands, timed on a bounded sample: `budget_rows` query rows against all n points."""
    import datagen
    from oracle import oracle as orc
    n, d = X.shape
    P = orc.decode(X)
    rows = datagen.query_rows(workload, budget_rows, n=n)
    t0 = time.perf_counter()
    rs, nbr, d2 = orc.rows_join(P, eps, rows)  # sizes, then fills: two passes over the sample
    dt = time.perf_counter() - t0
    evals = 2 * rows.size * (n - 1)
    return dict(value=2.0 * d * evals / dt / 1e12, unit="TFLOP/s", cores=orc.num_threads(), kind="oracle",
                sample=f"{rows.size} seeded query rows x all {n} points, FP64 difference form, evaluated twice (size pass + fill pass): "
                       f"{evals} distance evaluations in {dt:.2f} s; extrapolated full n(n-1)/2 join: {n * (n - 1) / 2 / (evals / dt):.0f} s",
                distance_evals_per_s=evals / dt)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", type=int, default=3, help="workload id 1..5 (datagen.WORKLOADS)")
    ap.add_argument("--selectivity", type=int, default=None)
    ap.add_argument("--mode", choices=["pairs", "count", "join", "split"], default="pairs",
                    help="pairs/count: self-join; join: two-set join of the workload's points against --queries query points; "
                         "split: higher-accuracy self-join of FP32 data (the workload's points plus seeded sub-FP16 noise), pair list")
    ap.add_argument("--queries", type=int, default=100_000, help="query points of --mode join (same distribution, rows n .. n+queries-1)")
    ap.add_argument("--power-probe", action="store_true",
                    help="also time the same shape on nearly-all-zero points (unique rows, two non-zero coordinates, epsilon 0): "
                         "operands that barely toggle the matrix cores, to separate the power limit from the kernel's structure")
    ap.add_argument("--graph", action="store_true", help="capture one step in a HIP graph and time replays (launch-bound small workloads)")
    ap.add_argument("--prepared", action="store_true", help="--mode join: prepare the point set once (ejoin_set), time the per-batch calls")
    ap.add_argument("--n", type=int, default=None, help="override the number of points (debugging)")
    ap.add_argument("--eps", type=float, default=None, help="override epsilon (0 = output-free run: isolates Gram + threshold from compaction)")
    ap.add_argument("--e2e", action="store_true", help="also time one end-to-end response: pinned host X -> HBM, step, found pairs -> pinned host")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=None)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one MI355X per box); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import datagen
    import paper_2508_21230_amd as pkg

    w = args.workload
    spec = datagen.WORKLOADS[w]
    S = args.selectivity or spec["selectivity"][0]
    n = args.n or spec["n"]
    d = spec["d"]
    eps = load_eps(w, S) if args.eps is None else args.eps
    nq = args.queries if args.mode == "join" else 0
    X = datagen.generate(w, n=n + nq)
    Xd = torch.from_numpy(X[:n].view(np.int16)).to("cuda:0")
    ej = pkg.EJoin(0)
    ej.reserve(n + nq, d)
    expect_pairs = int(n * (S / 2 * (n / spec["n"]) + 1)) if args.mode != "join" else int(nq * S * (n / spec["n"]) * 2)
    capacity = int(expect_pairs * 1.5) + (1 << 20)
    if args.mode == "split":
        ej.reserve(2 * n, 3 * ((d + 63) // 64 * 64))
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(datagen.data_seed(w))
        X32 = Xd.view(torch.float16).to(torch.float32)
        X32 += (torch.rand(X32.shape, generator=gen, device="cuda:0", dtype=torch.float32) - 0.5) * 2.0 ** -12
        pairs = torch.empty((capacity, 2), dtype=torch.int32, device="cuda:0")
        dist2 = torch.empty(capacity, dtype=torch.float32, device="cuda:0")
        npairs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        step = lambda: ej.selfjoin_pairs_f32(X32, eps, capacity, pairs=pairs, dist2=dist2, n_pairs=npairs)
    elif args.mode == "join":
        Qd = torch.from_numpy(np.ascontiguousarray(X[n:]).view(np.int16)).to("cuda:0")
        pairs = torch.empty((capacity, 2), dtype=torch.int32, device="cuda:0")
        dist2 = torch.empty(capacity, dtype=torch.float32, device="cuda:0")
        npairs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        if args.prepared:
            pset = ej.prepare(Xd)
            step = lambda: pset.join_pairs(Qd, eps, capacity, pairs=pairs, dist2=dist2, n_pairs=npairs)
        else:
            step = lambda: ej.join_pairs(Xd, Qd, eps, capacity, pairs=pairs, dist2=dist2, n_pairs=npairs)
    elif args.mode == "pairs":
        pairs = torch.empty((capacity, 2), dtype=torch.int32, device="cuda:0")
        dist2 = torch.empty(capacity, dtype=torch.float32, device="cuda:0")
        npairs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        step = lambda: ej.selfjoin_pairs(Xd, eps, capacity, pairs=pairs, dist2=dist2, n_pairs=npairs)
    else:
        counts = torch.empty(n, dtype=torch.int32, device="cuda:0")
        npairs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        step = lambda: ej.selfjoin_count(Xd, eps, counts=counts, total=npairs)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    join_ms, norm_ms = [], []
    if args.graph:
        # the library enqueues kernels only (workspace reserved above), so a step can be captured and replayed
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ej.set_profiling(True)  # kernel times from one eager step (events are not recorded inside a graph)
        step()
        a, b = ej.last_kernel_ms()
        norm_ms.append(a)
        join_ms.append(b)
        ej.set_profiling(False)
    else:
        ej.set_profiling(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
            a, b = ej.last_kernel_ms()  # waits for this step's events (HIP events on the launch stream)
            norm_ms.append(a)
            join_ms.append(b)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ej.set_profiling(False)
    found = int(npairs.cpu()[0])
    e2e = None
    if args.e2e and args.mode == "pairs":  # (not for the other modes)
        # End-to-end response time in the paper's sense (Section 4.1.1: transfers and result storage included).
        Xh = torch.from_numpy(X[:n].view(np.int16)).pin_memory()
        m = min(found, capacity)
        ph = torch.empty((m, 2), dtype=torch.int32).pin_memory()
        dh = torch.empty(m, dtype=torch.float32).pin_memory()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        Xd.copy_(Xh, non_blocking=True)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        m2 = min(int(npairs.cpu()[0]), m)
        ph[:m2].copy_(pairs[:m2], non_blocking=True)
        dh[:m2].copy_(dist2[:m2], non_blocking=True)
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        e2e = {"h2d_ms": (t2 - t1) * 1e3, "step_ms": (t3 - t2) * 1e3, "d2h_ms": (t4 - t3) * 1e3, "total_ms": (t4 - t1) * 1e3,
               "h2d_bytes": Xh.numel() * 2, "d2h_bytes": m2 * 12}
    ms_per_step = dt / args.steps * 1e3
    dk = (d + 63) // 64 * 64
    tiles = pkg.tiles_evaluated(n) if args.mode != "join" else pkg.tiles_evaluated2(n, nq)
    derived_flop = 2.0 * n * n * d if args.mode != "join" else 2.0 * n * nq * d
    flop_exec = 2.0 * 256 * 256 * dk * tiles * (3 if args.mode == "split" else 1)  # split: hi.hi + lo.hi + hi.lo
    jm = sum(join_ms) / len(join_ms)
    achieved = flop_exec / (jm * 1e-3) / 1e12
    emitted = found + (0 if args.mode == "pairs" else 0)
    out = {
        "metric": "self-join distance TFLOPS (2*n^2*d / t)" if args.mode != "join" else "two-set join distance TFLOPS (2*np*nq*d / t)",
        "value": derived_flop / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if args.mode != "split" else "f16x2 (split FP32)",
        "accumulate": "f32",
        "data": "synthetic",
        "hip_graph": bool(args.graph),
        "config": {"workload": f"configs[{w - 1}]: n={n}, d={d}, {spec['kind']}, S={S}, eps={eps:.7g}, mode={args.mode}",
                   "n": n, "d": d, "selectivity_target": S, "eps": eps, "mode": args.mode},
        "pairs_found": found,
        "pairs_per_s": emitted / (ms_per_step * 1e-3),
        "achieved_selectivity": (2.0 * (found - n) / n) if args.mode in ("pairs", "split") else (2.0 * found / n if args.mode == "count" else found / max(nq, 1)),
        "kernel_ms": {"norms": sum(norm_ms) / len(norm_ms), "join": jm, "join_min": min(join_ms), "join_median": sorted(join_ms)[len(join_ms) // 2]},
        "pairs_write_GBps": (min(found, capacity) * 12 / (jm * 1e-3) / 1e9) if args.mode != "count" else 0.0,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP16_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w, S, args.mode)) if args.n is None else None, "kernel": "k_join", "flop_per_launch": flop_exec, "tiles": tiles},
    }
    if args.mode == "join":
        out["config"]["queries"] = nq
        out["config"]["prepared_set"] = bool(args.prepared)
    if e2e is not None:
        out["end_to_end"] = e2e
    if args.power_probe and args.mode == "pairs":
        Z = torch.zeros((n, d), dtype=torch.float16, device="cuda:0")
        idx = torch.arange(n, device="cuda:0")
        Z[:, 0] = ((idx % 1024).float() / 1024).half()
        Z[:, 1] = ((idx // 1024).float() / 8192).half()
        Zi = Z.view(torch.int16)
        zstep = lambda: ej.selfjoin_pairs(Zi, 0.0, capacity, pairs=pairs, dist2=dist2, n_pairs=npairs)
        zstep()
        torch.cuda.synchronize()
        ej.set_profiling(True)
        zms = []
        for _ in range(max(2, args.steps)):
            zstep()
            zms.append(ej.last_kernel_ms()[1])
        ej.set_profiling(False)
        zt = sum(zms) / len(zms)
        out["power_probe"] = {"data": "near-zero points of the same shape, eps = 0", "join_ms": zt,
                              "achieved": flop_exec / (zt * 1e-3) / 1e12, "frac": flop_exec / (zt * 1e-3) / 1e12 / PEAK_FP16_TFLOPS}
    if not args.no_cpu_baseline and args.mode not in ("join", "split"):
        rows = args.cpu_rows or max(8, int(2.0e12 / (n * d * 16)))  # ~10-30 s of host work
        out["cpu_baseline"] = cpu_baseline(X[:n], w, eps, rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
