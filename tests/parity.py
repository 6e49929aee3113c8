"""Shared helpers of the GPU parity tests: the parity rule between the HIP path and the CPU oracle.

Rule (from the benchmark spec): the GPU pair set must equal the oracle's except for pairs whose
FP64 distance lies within a relative 1e-3 of epsilon; squared distances of common pairs must agree
within a relative 1e-3.  As D2 -> 0 an FP32 expansion s_i + s_j - 2a cannot hold a relative bound
(it cancels two numbers of size s), so the value tolerance is max(1e-3 * D2, 5e-7 * (s_i + s_j)):
the floor is about four FP32 ulps of the operands and only matters for near-duplicates.
"""
from __future__ import annotations

import numpy as np

from oracle import oracle as orc

REL = 1e-3
FLOOR = 5e-7


def to_host_pairs(pairs_t, d2_t, n_pairs_t):
    found = int(n_pairs_t.cpu()[0])
    cap = pairs_t.shape[0]
    m = min(found, cap)
    pairs = pairs_t[:m].cpu().numpy().view(np.uint32).reshape(m, 2)
    d2 = None if d2_t is None else d2_t[:m].cpu().numpy()
    return pairs, d2, found


def check_pair_sets(P, eps, gpu_pairs, gpu_d2, ora_pairs, ora_d2):
    """Asserts the parity rule; returns a dict of statistics (mismatch rate among boundary pairs etc.)."""
    n = P.shape[0]
    gp = np.asarray(gpu_pairs, dtype=np.uint32)
    assert gp.ndim == 2 and gp.shape[1] == 2
    assert (gp[:, 0] <= gp[:, 1]).all(), "pairs must have i <= j"
    assert gp.size == 0 or gp.max() < n, "index out of range"
    kg = orc.pair_keys(gp)
    order = np.argsort(kg, kind="stable")
    kg_sorted = kg[order]
    assert np.all(kg_sorted[1:] != kg_sorted[:-1]), "duplicate pairs in the GPU result"
    ko = orc.pair_keys(ora_pairs)  # sorted by construction
    assert np.all(ko[1:] > ko[:-1])
    # self pairs: all present on both sides
    assert (gp[:, 0] == gp[:, 1]).sum() == n and (ora_pairs[:, 0] == ora_pairs[:, 1]).sum() == n
    common_g = np.isin(kg_sorted, ko, assume_unique=True)
    common_o = np.isin(ko, kg_sorted, assume_unique=True)
    only_g = kg_sorted[~common_g]
    only_o_d2 = ora_d2[~common_o]
    # pairs only the oracle has must be boundary pairs
    assert orc.boundary_band(only_o_d2, eps, REL).all(), "GPU missed a pair outside the boundary band"
    # pairs only the GPU has: evaluate them with the oracle, must be boundary pairs
    if only_g.size:
        gi = (only_g >> np.uint64(32)).astype(np.int64)
        gj = (only_g & np.uint64(0xFFFFFFFF)).astype(np.int64)
        d2x = np.array([orc.dist2(P, i, j) for i, j in zip(gi, gj)])
        assert orc.boundary_band(d2x, eps, REL).all(), "GPU reported a pair outside the boundary band"
    stats = dict(pairs_gpu=int(gp.shape[0]), pairs_oracle=int(ora_pairs.shape[0]), only_gpu=int(only_g.size),
                 only_oracle=int(only_o_d2.size))
    band_total = int(orc.boundary_band(ora_d2, eps, REL).sum()) + int(only_g.size)
    stats["boundary_pairs"] = band_total
    stats["boundary_mismatch_rate"] = (only_g.size + only_o_d2.size) / band_total if band_total else 0.0
    if gpu_d2 is not None:
        g_d2 = np.asarray(gpu_d2)[order][common_g].astype(np.float64)
        o_d2 = ora_d2[common_o]
        s = orc.norms(P)
        op = ora_pairs[common_o]
        tol = np.maximum(REL * o_d2, FLOOR * (s[op[:, 0]] + s[op[:, 1]]))
        err = np.abs(g_d2 - o_d2)
        worst = int(np.argmax(err - tol))
        assert (err <= tol).all(), f"dist2 off: pair {op[worst]} gpu {g_d2[worst]} oracle {o_d2[worst]} tol {tol[worst]}"
        stats["floor_used"] = int((FLOOR * (s[op[:, 0]] + s[op[:, 1]]) > REL * o_d2).sum())
        nz = o_d2 > 0
        stats["max_rel_err_d2"] = float((err[nz] / o_d2[nz]).max()) if nz.any() else 0.0
        m, sd = orc.distance_error_stats(g_d2, o_d2)
        stats["dist_err_mean"], stats["dist_err_std"] = m, sd
    stats["overlap_accuracy"] = orc.overlap_accuracy(n, gp, ora_pairs)
    return stats


def check_rows(P, eps, rows, row_start, nbr, nd2, gpu_pairs, gpu_d2):
    """Neighbour lists of sampled query rows (oracle) against the full GPU pair list."""
    n = P.shape[0]
    gp = np.asarray(gpu_pairs, dtype=np.uint32)
    sel = np.zeros(n, dtype=bool)
    sel[rows] = True
    touching = sel[gp[:, 0]] | sel[gp[:, 1]]
    sub = gp[touching]
    subd = None if gpu_d2 is None else np.asarray(gpu_d2)[touching]
    mism = 0
    band = 0
    checked = 0
    s = orc.norms(P[rows])
    for r, q in enumerate(rows):
        a = sub[:, 0] == q
        b = sub[:, 1] == q
        got = np.concatenate([sub[a, 1], sub[b, 0]]).astype(np.int64)
        gd = None if subd is None else np.concatenate([subd[a], subd[b]])
        keep = got != q
        got = got[keep]
        if gd is not None:
            gd = gd[keep]
        want = nbr[row_start[r]:row_start[r + 1]].astype(np.int64)
        wd2 = nd2[row_start[r]:row_start[r + 1]]
        assert np.unique(got).size == got.size, "duplicate neighbour"
        only_o = ~np.isin(want, got)
        only_g = ~np.isin(got, want)
        assert orc.boundary_band(wd2[only_o], eps, REL).all(), f"row {q}: missed neighbours outside the band"
        if only_g.any():
            d2x = np.array([orc.dist2(P, q, j) for j in got[only_g]])
            assert orc.boundary_band(d2x, eps, REL).all(), f"row {q}: extra neighbours outside the band"
        mism += int(only_o.sum() + only_g.sum())
        band += int(orc.boundary_band(wd2, eps, REL).sum() + only_g.sum())
        if gd is not None and want.size:
            o = np.argsort(got)
            gs, gds = got[o], gd[o]
            pos = np.searchsorted(gs, want[~only_o])
            err = np.abs(gds[pos].astype(np.float64) - wd2[~only_o])
            sj = orc.norms(P[want[~only_o]])
            tol = np.maximum(REL * wd2[~only_o], FLOOR * (s[r] + sj))
            assert (err <= tol).all(), f"row {q}: dist2 off by {err.max()}"
            checked += int(err.size)
    return dict(rows=len(rows), boundary_pairs=band, mismatches=mism, d2_checked=checked)
