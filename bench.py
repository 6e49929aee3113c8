#!/usr/bin/env python3
"""Benchmark of the epsilon self-join hot path on one MI355X.

One "step" = one pass of the whole hot path over one synthetic workload that is already resident
in HBM: norms + re-layout, FP16 split of the norm terms, Gram + threshold + compaction kernel (pair
list with dist2, or per-point counts).  Prints ONE JSON line.

With no flags the line's headline is configs[3] of the benchmark spec (n = 2*10^6, d = 384, S = 16, pair list), the
larger of the two d >= 384 configurations the target is stated for, timed for --steps steps; `per_config`
then holds every configuration and mode of the benchmark spec (configs[0..4], configs[3] at its three
selectivities, configs[4] in pair and count mode), each timed for at least three steps with the shader
clock and socket power sampled while it ran.  `--workload W` times one configuration only (profiling runs).

`value` is the paper's derived throughput 2*n^2*d / t (Section 4.1.1: total operations of the all-pairs
comparison divided by the measured time), which credits the use of symmetry as speed; `roofline.achieved`
counts only the matrix-core work actually executed (upper-triangular 256x256 tiles) against the dense
FP16 MFMA peak, over the join kernel's own duration (HIP events on the launch stream).
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0  # MI355X dense FP16 MFMA, published
PEAK_CLOCK_MHZ = 2400.0
HEADLINE = (4, 16, "pairs")
# every configuration and mode the benchmark spec names: (workload id = configs index + 1, selectivity, mode)
ALL_CASES = [(1, 32, "pairs"), (2, 64, "pairs"), (3, 16, "pairs"), (4, 16, "pairs"), (4, 128, "pairs"), (4, 1024, "pairs"),
             (4, 1024, "count"), (5, 64, "pairs"), (5, 64, "count")]
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k_join_workload4_hbm_counters.txt")
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2508_21230_amd", "csrc", f) for f in ("ejoin.hip", "panel_layout.h", "tile_cursor.h")]


def load_eps(workload: int, S: int) -> float:
    with open(os.path.join(ROOT, "paper_2508_21230_amd", "workloads_eps.json")) as f:
        return float(json.load(f)[str(workload)]["eps"][str(S)]["eps"])


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for p in KERNEL_SOURCES:
        h.update(open(p, "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(case):
    """Memory-side bytes of k_join per launch from the rocprofv3 --pmc summary under profiles/ -- only if that summary
    was taken on the headline case with the kernel source as it is now (its hash is part of the file); else None."""
    if case != HEADLINE or not os.path.exists(TRAFFIC_FILE):
        return None, None
    text = open(TRAFFIC_FILE).read()
    m = re.search(r"traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", text)
    k = re.search(r"kernel_source_sha256_16\s*=\s*([0-9a-f]{16})", text)
    if not m or not k or k.group(1) != kernel_source_hash():
        return None, None
    return float(m.group(1)), os.path.relpath(TRAFFIC_FILE, ROOT)


class ClockPowerSampler:
    """Samples the shader clock and the socket power from sysfs while a case runs (the paper's profiler table
    has a clock row for the same reason, Section 4.4: sustained matrix-core work is power-throttled)."""

    def __init__(self, period_s: float = 0.02):
        self.period = period_s
        self.sclk, self.power = [], []
        self.cap_w = None
        self._stop = threading.Event()
        self._thread = None
        devs = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.sclk_path = devs[0] if devs else None
        hw = sorted(glob.glob(os.path.dirname(self.sclk_path) + "/hwmon/hwmon*")) if self.sclk_path else []
        self.power_path = next((os.path.join(h, "power1_input") for h in hw if os.path.exists(os.path.join(h, "power1_input"))), None)
        cap = next((os.path.join(h, "power1_cap") for h in hw if os.path.exists(os.path.join(h, "power1_cap"))), None)
        try:
            self.cap_w = int(open(cap).read()) / 1e6 if cap else None
        except (OSError, ValueError):
            pass

    def _run(self):
        while not self._stop.is_set():
            try:
                if self.sclk_path:
                    m = re.search(r"(\d+)\s*Mhz\s*\*", open(self.sclk_path).read())
                    if m:
                        self.sclk.append(int(m.group(1)))
                if self.power_path:
                    self.power.append(int(open(self.power_path).read()) / 1e6)
            except (OSError, ValueError):
                pass
            self._stop.wait(self.period)

    def __enter__(self):
        self._thread = threading.Thread(target=self._run, daemon=True)
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join()

    def summary(self):
        out = {"samples": len(self.sclk), "power_cap_W": self.cap_w}
        if self.sclk:
            out.update(sclk_MHz_mean=sum(self.sclk) / len(self.sclk), sclk_MHz_min=min(self.sclk), sclk_MHz_max=max(self.sclk))
        if self.power:
            out.update(power_W_mean=sum(self.power) / len(self.power), power_W_max=max(self.power))
        return out


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
                sample=f"configs[{workload - 1}]: {rows.size} seeded query rows x all {n} points, FP64 difference form, evaluated twice "
                       f"(size pass + fill pass): {evals} distance evaluations in {dt:.2f} s; extrapolated full n(n-1)/2 join: "
                       f"{n * (n - 1) / 2 / (evals / dt):.0f} s",
                distance_evals_per_s=evals / dt)


class Case:
    """One configuration resident on the GPU, with a `step` callable that runs the hot path once."""

    def __init__(self, ej, w, S, mode, n=None, eps=None, queries=0, prepared=False, X=None):
        import numpy as np
        import torch

        import datagen
        spec = datagen.WORKLOADS[w]
        self.w, self.S, self.mode, self.spec = w, S, mode, spec
        self.n = n or spec["n"]
        self.d = spec["d"]
        self.eps = load_eps(w, S) if eps is None else eps
        self.nq = queries if mode == "join" else 0
        n, nq, d = self.n, self.nq, self.d
        self.X = X if X is not None else datagen.generate(w, n=n + nq)
        self.Xd = torch.from_numpy(self.X[:n].view(np.int16)).to("cuda:0")
        ej.reserve(n + nq, d)
        scale = n / spec["n"]
        expect = int(n * (S / 2 * scale + 1)) if mode != "join" else int(nq * S * scale * 2)
        self.capacity = cap = int(expect * 1.5) + (1 << 20)
        dev = "cuda:0"
        self.npairs = torch.zeros(1, dtype=torch.int64, device=dev)
        if mode == "count":
            self.counts = torch.empty(n, dtype=torch.int32, device=dev)
            self.step = lambda: ej.selfjoin_count(self.Xd, self.eps, counts=self.counts, total=self.npairs)
            return
        self.pairs = torch.empty((cap, 2), dtype=torch.int32, device=dev)
        self.dist2 = torch.empty(cap, dtype=torch.float32, device=dev)
        out = dict(pairs=self.pairs, dist2=self.dist2, n_pairs=self.npairs)
        if mode == "split":
            ej.reserve(2 * n, 3 * ((d + 63) // 64 * 64))
            gen = torch.Generator(device=dev)
            gen.manual_seed(datagen.data_seed(w))
            self.X32 = self.Xd.view(torch.float16).to(torch.float32)
            self.X32 += (torch.rand(self.X32.shape, generator=gen, device=dev, dtype=torch.float32) - 0.5) * 2.0 ** -12
            self.step = lambda: ej.selfjoin_pairs_f32(self.X32, self.eps, cap, **out)
        elif mode == "join":
            self.Qd = torch.from_numpy(np.ascontiguousarray(self.X[n:]).view(np.int16)).to(dev)
            if prepared:
                self.pset = ej.prepare(self.Xd)
                self.step = lambda: self.pset.join_pairs(self.Qd, self.eps, cap, **out)
            else:
                self.step = lambda: ej.join_pairs(self.Xd, self.Qd, self.eps, cap, **out)
        else:
            self.step = lambda: ej.selfjoin_pairs(self.Xd, self.eps, cap, **out)

    def label(self):
        return (f"configs[{self.w - 1}]: n={self.n}, d={self.d}, {self.spec['kind']}, S={self.S}, eps={self.eps:.7g}, mode={self.mode}")

    def flops(self, pkg):
        dk = (self.d + 63) // 64 * 64
        tiles = pkg.tiles_evaluated(self.n) if self.mode != "join" else pkg.tiles_evaluated2(self.n, self.nq)
        derived = 2.0 * self.n * self.n * self.d if self.mode != "join" else 2.0 * self.n * self.nq * self.d
        executed = 2.0 * 256 * 256 * dk * tiles * (3 if self.mode == "split" else 1)  # split: hi.hi + lo.hi + hi.lo
        return derived, executed, tiles


def time_case(ej, pkg, case, steps, warmup, graph=False):
    """Times `steps` steps after `warmup`; returns the measurements of one configuration."""
    import torch
    for _ in range(warmup):
        case.step()
    torch.cuda.synchronize()
    join_ms, prep_ms = [], []
    with ClockPowerSampler() as sampler:
        if graph:
            # the library enqueues kernels only (workspace reserved), so a step can be captured and replayed
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                case.step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                case.step()
            g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                g.replay()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            ej.set_profiling(True)  # kernel times from one eager step (events are not recorded inside a graph)
            case.step()
            a, b = ej.last_kernel_ms()
            prep_ms.append(a)
            join_ms.append(b)
            ej.set_profiling(False)
        else:
            dt_plain = None
            if _estimate_s(case) < 5e-3:
                # short steps: the per-step wait for the kernel events would dominate, so the step time comes from a
                # loop of its own that only enqueues; the loop with events below then gives the kernel times
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    case.step()
                torch.cuda.synchronize()
                dt_plain = time.perf_counter() - t0
            ej.set_profiling(True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                case.step()
                a, b = ej.last_kernel_ms()  # waits for this step's events (HIP events on the launch stream)
                prep_ms.append(a)
                join_ms.append(b)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            ej.set_profiling(False)
            if dt_plain is not None:
                dt = dt_plain
    found = int(case.npairs.cpu()[0])
    ms = dt / steps * 1e3
    jm = sum(join_ms) / len(join_ms)
    derived, executed, tiles = case.flops(pkg)
    achieved = executed / (jm * 1e-3) / 1e12
    n, nq, mode = case.n, case.nq, case.mode
    clk = sampler.summary()
    res = {
        "workload": case.label(), "mode": mode, "selectivity_target": case.S, "eps": case.eps, "steps": steps, "ms_per_step": ms,
        "value": derived / (ms * 1e-3) / 1e12,
        "kernel_ms": {"prep": sum(prep_ms) / len(prep_ms), "join": jm, "join_min": min(join_ms), "join_median": sorted(join_ms)[len(join_ms) // 2]},
        "achieved": achieved, "frac": achieved / PEAK_FP16_TFLOPS,
        "pairs_found": found, "pairs_per_s": found / (ms * 1e-3),
        "achieved_selectivity": (2.0 * (found - n) / n) if mode in ("pairs", "split") else (2.0 * found / n if mode == "count" else found / max(nq, 1)),
        "pair_store_GBps": (min(found, case.capacity) * 12 / (jm * 1e-3) / 1e9) if mode != "count" else 0.0,
        "clock_power": clk, "tiles": tiles, "flop_per_launch": executed,
    }
    if clk.get("sclk_MHz_mean"):
        # the same work against the peak the chip would have at the clock it actually ran at
        res["frac_at_measured_clock"] = achieved / (PEAK_FP16_TFLOPS * clk["sclk_MHz_mean"] / PEAK_CLOCK_MHZ)
    return res


def calibrate_counters():
    """A plain device-to-device copy of known size (4 GiB read, 4 GiB written), for scaling FETCH_SIZE / WRITE_SIZE of a
    rocprofv3 --pmc run: what the counters read for this copy kernel gives the bytes one count stands for."""
    import torch
    n = 1 << 30
    a = torch.arange(n, dtype=torch.int32, device="cuda:0")
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    b.copy_(a)
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "device copy", "bytes_read": 4 * n, "bytes_written": 4 * n, "check": int(b[12345].item())}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", type=int, default=None,
                    help="time only this workload id 1..5 (datagen.WORKLOADS; id = configs index + 1); default: the headline and every configuration")
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
    ap.add_argument("--calibrate-counters", action="store_true", help="run one 4 GiB device copy and exit (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one MI355X per box); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_counters:
        calibrate_counters()
        return

    import numpy as np
    import torch

    import datagen
    import paper_2508_21230_amd as pkg

    ej = pkg.EJoin(0)
    single = args.workload is not None
    hw, hS, hmode = (args.workload, args.selectivity or datagen.WORKLOADS[args.workload]["selectivity"][0], args.mode) if single else HEADLINE
    head_case = Case(ej, hw, hS, hmode, n=args.n, eps=args.eps, queries=args.queries, prepared=args.prepared)
    head = time_case(ej, pkg, head_case, args.steps, args.warmup, graph=args.graph)
    traffic, traffic_source = measured_traffic((hw, hS, hmode)) if (args.n is None and args.eps is None) else (None, None)
    out = {
        "metric": "self-join distance TFLOPS (2*n^2*d / t)" if hmode != "join" else "two-set join distance TFLOPS (2*np*nq*d / t)",
        "value": head["value"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if hmode != "split" else "f16x2 (split FP32)",
        "accumulate": "f32",
        "data": "synthetic",
        "hip_graph": bool(args.graph),
        "config": {"workload": head["workload"], "n": head_case.n, "d": head_case.d, "selectivity_target": hS, "eps": head_case.eps, "mode": hmode},
        "pairs_found": head["pairs_found"],
        "pairs_per_s": head["pairs_per_s"],
        "achieved_selectivity": head["achieved_selectivity"],
        "kernel_ms": head["kernel_ms"],
        "pairs_write_GBps": head["pair_store_GBps"],
        "clock_power": head["clock_power"],
        "roofline": {"bound": "mfma", "achieved": head["achieved"], "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s", "frac": head["frac"],
                     "frac_at_measured_clock": head.get("frac_at_measured_clock"),
                     "traffic": traffic, "traffic_source": traffic_source, "kernel": "k_join", "flop_per_launch": head["flop_per_launch"],
                     "tiles": head["tiles"]},
    }
    if hmode == "join":
        out["config"]["queries"] = head_case.nq
        out["config"]["prepared_set"] = bool(args.prepared)

    if args.e2e and hmode == "pairs":
        # End-to-end response time in the paper's sense (Section 4.1.1: transfers and result storage included).
        c = head_case
        Xh = torch.from_numpy(c.X[:c.n].view(np.int16)).pin_memory()
        m = min(head["pairs_found"], c.capacity)
        ph = torch.empty((m, 2), dtype=torch.int32).pin_memory()
        dh = torch.empty(m, dtype=torch.float32).pin_memory()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        c.Xd.copy_(Xh, non_blocking=True)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        c.step()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        m2 = min(int(c.npairs.cpu()[0]), m)
        ph[:m2].copy_(c.pairs[:m2], non_blocking=True)
        dh[:m2].copy_(c.dist2[:m2], non_blocking=True)
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        out["end_to_end"] = {"h2d_ms": (t2 - t1) * 1e3, "step_ms": (t3 - t2) * 1e3, "d2h_ms": (t4 - t3) * 1e3, "total_ms": (t4 - t1) * 1e3,
                             "h2d_bytes": Xh.numel() * 2, "d2h_bytes": m2 * 12}
        # the same response with the result returned in batches while the join runs (ejoin_selfjoin_pairs_to_host)
        for nb in (4, 16):
            torch.cuda.synchronize()
            t5 = time.perf_counter()
            c.Xd.copy_(Xh, non_blocking=True)
            got = ej.selfjoin_pairs_to_host(c.Xd, c.eps, nb, c.pairs[:m], c.dist2[:m], ph, dh)
            t6 = time.perf_counter()
            assert got == head["pairs_found"]
            out["end_to_end"][f"batched_{nb}_total_ms"] = (t6 - t5) * 1e3
    if args.power_probe and hmode == "pairs":
        c = head_case
        Z = torch.zeros((c.n, c.d), dtype=torch.float16, device="cuda:0")
        idx = torch.arange(c.n, device="cuda:0")
        Z[:, 0] = ((idx % 1024).float() / 1024).half()
        Z[:, 1] = ((idx // 1024).float() / 8192).half()
        Zi = Z.view(torch.int16)
        zstep = lambda: ej.selfjoin_pairs(Zi, 0.0, c.capacity, pairs=c.pairs, dist2=c.dist2, n_pairs=c.npairs)
        zstep()
        torch.cuda.synchronize()
        ej.set_profiling(True)
        zms = []
        with ClockPowerSampler() as zs:
            for _ in range(max(2, args.steps)):
                zstep()
                zms.append(ej.last_kernel_ms()[1])
        ej.set_profiling(False)
        zt = sum(zms) / len(zms)
        out["power_probe"] = {"data": "near-zero points of the same shape, eps = 0", "join_ms": zt,
                              "achieved": head["flop_per_launch"] / (zt * 1e-3) / 1e12,
                              "frac": head["flop_per_launch"] / (zt * 1e-3) / 1e12 / PEAK_FP16_TFLOPS, "clock_power": zs.summary()}

    cpu_X = head_case.X[:head_case.n] if (not args.no_cpu_baseline and hmode in ("pairs", "count")) else None
    cpu_eps, cpu_n, cpu_d = head_case.eps, head_case.n, head_case.d
    if not single:
        # every configuration and mode of the benchmark spec, the headline's own line first
        per = []
        cache = {hw: head_case.X}
        del head_case
        torch.cuda.empty_cache()
        for (w, S, mode) in ALL_CASES:
            if (w, S, mode) == HEADLINE:
                r = dict(head)
            else:
                if w not in cache:
                    cache.clear()
                    cache[w] = datagen.generate(w)
                c = Case(ej, w, S, mode, X=cache[w])
                # small workloads: enough steps for a stable mean (a step of configs[0] is tens of microseconds)
                steps = max(3, min(200, int(0.25 / max(1e-5, _estimate_s(c)))))
                r = time_case(ej, pkg, c, steps, 1)
                del c
                torch.cuda.empty_cache()
            print(f"[bench] {r['workload']}: {r['ms_per_step']:.3f} ms/step, frac {r['frac']:.3f}", file=sys.stderr, flush=True)
            per.append(r)
        out["per_config"] = per
    if cpu_X is not None:
        rows = args.cpu_rows or max(8, int(2.0e12 / (cpu_n * cpu_d * 16)))  # ~10-30 s of host work
        out["cpu_baseline"] = cpu_baseline(cpu_X, hw, cpu_eps, rows)
    print(json.dumps(out))


def _estimate_s(case) -> float:
    """Rough duration of one step, to pick a step count for the short workloads (1.2 PFLOP/s executed, 40 us floor)."""
    dk = (case.d + 63) // 64 * 64
    return max(4e-5, case.n * case.n * dk / 1.2e15)


if __name__ == "__main__":
    main()
