"""Seeded synthetic inputs for the epsilon self-join workloads.

This module only draws random numbers and rounds them to fp16; it holds none of the
join's arithmetic (no distances, no norms, no thresholds), so both the CPU oracle and
the HIP path may take their inputs from it.

The five workloads stand in for the data sets of the paper's evaluation (Section 4.1,
Table "datasets": Sift10M d=128, Tiny5M d=384, Gist1M d=960, Synth |D|=1e5), borrowing
their shapes only: values here are uniform or clipped Gaussian mixtures in [0, 1].

Recipe (identical bytes on every machine for a given workload id and n):
  * rows are produced in chunks of CHUNK_ROWS; chunk c of workload w draws from
    numpy Generator(Philox(key=[data_seed(w), c])), so any chunk can be regenerated alone;
  * "uniform": x = U[0,1) drawn in fp32;
  * "mixture": cluster centres U[0,1)^d in fp32 from Philox(key=[data_seed(w), 2**63]);
    each row draws its cluster id uniformly, then x = centre + sigma * N(0,1) in fp32,
    clipped to [0, 1];
  * the fp32 values are rounded once to fp16 (round-to-nearest-even, numpy astype) and
    returned as uint16 bit patterns, row-major, shape (n, d).
"""
from __future__ import annotations

import concurrent.futures as _cf
import os as _os

import numpy as np

CHUNK_ROWS = 65536

#: workload id -> description.  `selectivity` lists the mean neighbours/point targets.
WORKLOADS = {
    1: dict(n=4096, d=128, kind="uniform", selectivity=(32,), eps_from="all_pairs"),
    2: dict(n=100_000, d=128, kind="mixture", clusters=100, sigma=0.05, selectivity=(64,), eps_from="sample"),
    3: dict(n=1_000_000, d=960, kind="mixture", clusters=1_000, sigma=0.02, selectivity=(16,), eps_from="sample"),
    4: dict(n=2_000_000, d=384, kind="mixture", clusters=2_000, sigma=0.03, selectivity=(16, 128, 1024), eps_from="sample"),
    5: dict(n=5_000_000, d=128, kind="mixture", clusters=10_000, sigma=0.05, selectivity=(64,), eps_from="sample"),
    # not one of the task's five configurations: a scale test (1.1e9 tiles, two data slices per tile)
    6: dict(n=12_000_000, d=64, kind="mixture", clusters=20_000, sigma=0.05, selectivity=(64,), eps_from="sample"),
}

SAMPLE_POINTS = 2048


def data_seed(workload: int) -> int:
    return 1000 + workload


def sample_seed(workload: int) -> int:
    return 2000 + workload


def _centres(workload: int) -> np.ndarray:
    w = WORKLOADS[workload]
    rng = np.random.Generator(np.random.Philox(key=np.array([data_seed(workload), 2**63], dtype=np.uint64)))
    return rng.random((w["clusters"], w["d"]), dtype=np.float32)


def _chunk(workload: int, c: int, rows: int, centres) -> np.ndarray:
    w = WORKLOADS[workload]
    d = w["d"]
    rng = np.random.Generator(np.random.Philox(key=np.array([data_seed(workload), c], dtype=np.uint64)))
    if w["kind"] == "uniform":
        x = rng.random((CHUNK_ROWS, d), dtype=np.float32)[:rows]
    else:
        ids = rng.integers(0, w["clusters"], size=CHUNK_ROWS)[:rows]
        # the noise is drawn for the rows actually used only; a chunk's content depends on
        # (workload, c, rows-in-chunk), and rows-in-chunk is fixed by n
        x = rng.standard_normal((rows, d), dtype=np.float32)
        x *= np.float32(w["sigma"])
        x += centres[ids]
        np.clip(x, 0.0, 1.0, out=x)
    return x.astype(np.float16).view(np.uint16)


def generate(workload: int, n: int | None = None, out: np.ndarray | None = None, threads: int | None = None) -> np.ndarray:
    """Return the (n, d) uint16 array of fp16 bit patterns of a workload.

    `n` smaller than the workload's own size gives a prefix-compatible scaled-down data set
    only for full chunks; tests that need small inputs simply use the small n as its own
    data set (same distribution, same seed).
    """
    w = WORKLOADS[workload]
    n = w["n"] if n is None else int(n)
    d = w["d"]
    if out is None:
        out = np.empty((n, d), dtype=np.uint16)
    assert out.shape == (n, d) and out.dtype == np.uint16
    centres = _centres(workload) if w["kind"] == "mixture" else None
    nchunks = (n + CHUNK_ROWS - 1) // CHUNK_ROWS

    def work(c):
        r0 = c * CHUNK_ROWS
        rows = min(CHUNK_ROWS, n - r0)
        out[r0:r0 + rows] = _chunk(workload, c, rows, centres)

    if threads is None:
        threads = min(16, _os.cpu_count() or 1)
    if nchunks == 1 or threads <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with _cf.ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunks)))
    return out


def sample_indices(workload: int, n: int | None = None, m: int = SAMPLE_POINTS) -> np.ndarray:
    """m distinct row indices (sorted) drawn with the workload's sample seed."""
    n = WORKLOADS[workload]["n"] if n is None else int(n)
    m = min(m, n)
    rng = np.random.Generator(np.random.Philox(key=np.array([sample_seed(workload), 0], dtype=np.uint64)))
    return np.sort(rng.choice(n, size=m, replace=False)).astype(np.int64)


def query_rows(workload: int, count: int, n: int | None = None) -> np.ndarray:
    """`count` distinct row indices (sorted) used by sampled parity checks and the CPU baseline."""
    n = WORKLOADS[workload]["n"] if n is None else int(n)
    count = min(count, n)
    rng = np.random.Generator(np.random.Philox(key=np.array([sample_seed(workload), 1], dtype=np.uint64)))
    return np.sort(rng.choice(n, size=count, replace=False)).astype(np.int64)


def lattice_points(n: int, d: int, h: float) -> np.ndarray:
    """Points x_t = t*h*e_1 (t = 0..n-1) as fp16 bits; h and every t*h must be fp16-exact."""
    x = np.zeros((n, d), dtype=np.float32)
    x[:, 0] = np.arange(n, dtype=np.float32) * np.float32(h)
    h16 = x.astype(np.float16)
    assert np.array_equal(h16.astype(np.float32), x), "lattice coordinates must be exact in fp16"
    return h16.view(np.uint16)
