"""Full-size parity of the five workloads of the benchmark spec: shared by tests/test_gpu_fullsize.py and by
tests/parity_full_size_record.py (which writes the per-workload accuracy record).

A workload is generated once, joined by the GPU at each of its selectivities in the launch configuration
bench.py times, and held against the oracle under the STRICT parity rule (tests/parity.py, strict=True:
relative 1e-3 band and relative 1e-3 value tolerance only, no floors):
  * workloads 1 and 2 are joined in full by the oracle;
  * workloads 3-5 on seeded query rows: the oracle's exact neighbour lists of those rows (one pass at the
    workload's largest epsilon, cut down to each smaller epsilon by the same `D2 <= eps^2` comparison)
    against the neighbours the GPU pair list holds for them;
  * whole-output properties that hold at any size: i <= j, indices in range, no duplicate pair, every
    self pair present, count mode == histogram of pair mode.
"""
from __future__ import annotations

import functools
import json
import os
import time

import numpy as np
import torch

import datagen
from oracle import oracle as orc
from tests import parity

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROW_CHUNK = 256  # query rows per oracle call (a progress line after each)


def stored_eps(w, S):
    return float(json.load(open(os.path.join(ROOT, "paper_2508_21230_amd", "workloads_eps.json")))[str(w)]["eps"][str(S)]["eps"])


def gpu_pair_properties(pairs_t, found, n):
    """Whole-output checks on the device (the lists are too long for numpy on the host)."""
    p = pairs_t[:found].to(torch.int64) & 0xFFFFFFFF
    i, j = p[:, 0], p[:, 1]
    assert bool((i <= j).all()) and int(j.max()) < n
    assert int((i == j).sum()) == n, "every self pair exactly once"
    keys = (i << 32) | j
    assert int(torch.unique(keys).numel()) == found, "duplicate pairs"
    return i, j


@functools.lru_cache(maxsize=1)
def oracle_side(w, rows):
    """The workload's bytes, their FP64 decoding and the oracle's result at the workload's LARGEST epsilon:
    rows=None -> the full join (pairs, D2), else the neighbour lists of `rows` seeded query rows."""
    spec = datagen.WORKLOADS[w]
    t0 = time.time()
    X = datagen.generate(w)
    P = orc.decode(X)
    print(f"\nworkload {w}: n={spec['n']} d={spec['d']} generated and decoded in {time.time() - t0:.1f}s", flush=True)
    eps_max = max(stored_eps(w, S) for S in spec["selectivity"])
    t0 = time.time()
    if rows is None:
        pairs, d2 = orc.selfjoin_pairs(P, eps_max)
        print(f"  oracle: full join, {pairs.shape[0]} pairs in {time.time() - t0:.1f}s", flush=True)
        return X, P, ("full", pairs, d2)
    q = datagen.query_rows(w, rows)
    starts, nbrs, d2s = [np.zeros(1, dtype=np.int64)], [], []
    for c in range(0, q.size, ROW_CHUNK):
        rs, nb, dd = orc.rows_join(P, eps_max, q[c:c + ROW_CHUNK])
        starts.append(rs[1:] + starts[-1][-1])
        nbrs.append(nb)
        d2s.append(dd)
        print(f"  oracle: {min(c + ROW_CHUNK, q.size)}/{q.size} query rows x {spec['n']} points, {time.time() - t0:.1f}s", flush=True)
    return X, P, ("rows", q, np.concatenate(starts), np.concatenate(nbrs), np.concatenate(d2s))


def cut_to_eps(row_start, nbr, d2, eps):
    """Neighbour lists at a smaller epsilon: the entries with D2 <= eps^2 (the oracle's own comparison)."""
    keep = d2 <= orc.eps2_of(eps)
    per_row = np.add.reduceat(keep.astype(np.int64), row_start[:-1]) if keep.size else np.zeros(row_start.size - 1, dtype=np.int64)
    per_row[np.diff(row_start) == 0] = 0  # reduceat repeats the next segment for an empty one
    rs = np.concatenate([[0], np.cumsum(per_row)])
    return rs, nbr[keep], d2[keep]


def check_workload(ej, w, S, rows):
    """GPU self-join of workload w at selectivity S against the oracle (see the module text); returns statistics."""
    spec = datagen.WORKLOADS[w]
    n, d = spec["n"], spec["d"]
    eps = stored_eps(w, S)
    X, P, ora = oracle_side(w, rows)
    Xd = torch.from_numpy(X.view(np.int16)).cuda()
    capacity = int(n * (S / 2 + 1) * 1.6) + (1 << 20)
    pairs, d2, npairs = ej.selfjoin_pairs(Xd, eps, capacity)
    torch.cuda.synchronize()
    assert ej.status() == 0
    found = int(npairs.cpu()[0])
    assert found <= capacity
    print(f"  workload {w} S={S} eps={eps:.6g}: gpu join found {found} pairs, achieved selectivity {2 * (found - n) / n:.2f}", flush=True)
    i, j = gpu_pair_properties(pairs, found, n)
    # count mode agrees with the pair list
    counts, total = ej.selfjoin_count(Xd, eps)
    torch.cuda.synchronize()
    ns = i != j
    hist = torch.bincount(i[ns], minlength=n) + torch.bincount(j[ns], minlength=n)
    assert int(total.cpu()[0]) == found - n
    assert bool((hist == (counts.to(torch.int64) & 0xFFFFFFFF)).all())
    del hist, ns, counts
    if ora[0] == "full":
        _, opairs, od2 = ora
        keep = od2 <= orc.eps2_of(eps)
        hp, hd2, _ = parity.to_host_pairs(pairs, d2, npairs)
        st = parity.check_pair_sets(P, eps, hp, hd2, opairs[keep], od2[keep], strict=True)
        st["checked"] = "oracle join of all n points"
        st["d2_checked"] = st["pairs_oracle"] - st["only_oracle"]
    else:
        _, q, rs, nbr, nd2 = ora
        sel = torch.zeros(n, dtype=torch.bool, device="cuda")
        sel[torch.from_numpy(q).cuda()] = True
        touch = sel[i] | sel[j]
        sub = torch.stack([i[touch], j[touch]], 1).cpu().numpy().astype(np.uint32)
        subd = d2[:found][touch].cpu().numpy()
        rs_e, nbr_e, nd2_e = cut_to_eps(rs, nbr, nd2, eps)
        st = parity.check_rows(P, eps, q, rs_e, nbr_e, nd2_e, sub, subd, strict=True)
        st["checked"] = f"{q.size} seeded query rows x all n points"
    del pairs, d2, i, j, Xd
    torch.cuda.empty_cache()
    st.update(workload=w, n=n, d=d, selectivity_target=S, eps=eps, pairs_found=found, achieved_selectivity=2 * (found - n) / n)
    print("  ", st, flush=True)
    return st
