"""Parity at the full sizes of the five workloads, in the launch configuration bench.py times.

The oracle cannot join millions of points, so each workload is checked on
  * seeded query rows: their exact FP64 neighbour lists against the neighbours the GPU pair list
    holds for them (parity rule of tests/parity.py, squared distances included);
  * properties of the whole GPU output that hold at any size: i <= j, indices in range, no
    duplicate pair, every self pair present, count mode == histogram of pair mode.
"""
import json
import os
import time

import numpy as np
import pytest
import torch

import datagen
from oracle import oracle as orc
from tests import parity

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def stored_eps(w, S):
    return float(json.load(open(os.path.join(ROOT, "paper_2508_21230_amd", "workloads_eps.json")))[str(w)]["eps"][str(S)]["eps"])


@pytest.fixture(scope="module")
def ej():
    import paper_2508_21230_amd as pkg
    e = pkg.EJoin(0)
    yield e
    e.close()


def gpu_pair_properties(pairs_t, found, n):
    """Whole-output checks on the device (the lists are too long for numpy on the host)."""
    p = pairs_t[:found].to(torch.int64) & 0xFFFFFFFF
    i, j = p[:, 0], p[:, 1]
    assert bool((i <= j).all()) and int(j.max()) < n
    assert int((i == j).sum()) == n, "every self pair exactly once"
    keys = (i << 32) | j
    assert int(torch.unique(keys).numel()) == found, "duplicate pairs"
    return i, j


# workload 6 is not one of the task's configurations: 12 M points at d = 64 (1.1e9 tiles, exactly as many slices
# per tile as the copy pipeline runs ahead) as a test of scale
@pytest.mark.parametrize("w,S,rows", [(2, 64, 256), (3, 16, 48), (4, 16, 64), (4, 128, 64), (4, 1024, 16), (5, 64, 96), (6, 64, 32)])
def test_full_size_pairs_against_oracle_rows(ej, w, S, rows):
    spec = datagen.WORKLOADS[w]
    n, d = spec["n"], spec["d"]
    eps = stored_eps(w, S)
    t0 = time.time()
    X = datagen.generate(w)
    print(f"\nworkload {w} S={S}: generated n={n} d={d} in {time.time() - t0:.1f}s", flush=True)
    Xd = torch.from_numpy(X.view(np.int16)).cuda()
    capacity = int(n * (S / 2 + 1) * 1.6) + (1 << 20)
    pairs, d2, npairs = ej.selfjoin_pairs(Xd, eps, capacity)
    torch.cuda.synchronize()
    assert ej.status() == 0
    found = int(npairs.cpu()[0])
    assert found <= capacity
    print(f"  gpu join done: {found} pairs, achieved selectivity {2 * (found - n) / n:.2f}", flush=True)
    i, j = gpu_pair_properties(pairs, found, n)
    # count mode agrees with the pair list
    counts, total = ej.selfjoin_count(Xd, eps)
    torch.cuda.synchronize()
    ns = i != j
    hist = torch.bincount(i[ns], minlength=n) + torch.bincount(j[ns], minlength=n)
    assert int(total.cpu()[0]) == found - n
    assert bool((hist == (counts.to(torch.int64) & 0xFFFFFFFF)).all())
    # sampled query rows against the oracle
    q = datagen.query_rows(w, rows)
    sel = torch.zeros(n, dtype=torch.bool, device="cuda")
    sel[torch.from_numpy(q).cuda()] = True
    touch = sel[i] | sel[j]
    sub = torch.stack([i[touch], j[touch]], 1).cpu().numpy().astype(np.uint32)
    subd = d2[:found][touch].cpu().numpy()
    del pairs, d2, i, j, touch, hist, Xd
    torch.cuda.empty_cache()
    t0 = time.time()
    P = orc.decode(X)
    rs, nbr, nd2 = orc.rows_join(P, eps, q)
    print(f"  oracle: {rows} query rows x {n} points in {time.time() - t0:.1f}s, {nbr.size} neighbours", flush=True)
    st = parity.check_rows(P, eps, q, rs, nbr, nd2, sub, subd)
    print("  ", st, flush=True)
    assert st["d2_checked"] > 0


def test_full_size_two_set_join_against_oracle_queries(ej):
    """bench.py --mode join at its full size: the 10^6 points of workload 3 against 10^5 query points; 40 sampled
    query points are joined exactly by the oracle, the whole output is checked for range, duplicates and counts."""
    from tests.test_gpu_twoset import check_two_set
    w, n, nq = 3, datagen.WORKLOADS[3]["n"], 100_000
    eps = stored_eps(w, 16)
    X = datagen.generate(w, n=n + nq)
    Pd = torch.from_numpy(X[:n].view(np.int16)).cuda()
    Qd = torch.from_numpy(np.ascontiguousarray(X[n:]).view(np.int16)).cuda()
    cap = 8_000_000
    pairs, d2, npairs = ej.join_pairs(Pd, Qd, eps, cap)
    torch.cuda.synchronize()
    assert ej.status() == 0
    found = int(npairs.cpu()[0])
    assert 0 < found <= cap
    p = pairs[:found].to(torch.int64) & 0xFFFFFFFF
    i, j = p[:, 0], p[:, 1]
    assert int(i.max()) < n and int(j.max()) < nq
    assert int(torch.unique((i << 32) | j).numel()) == found
    cp, cq, total = ej.join_count(Pd, Qd, eps)
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == found
    assert bool((torch.bincount(i, minlength=n) == (cp.to(torch.int64) & 0xFFFFFFFF)).all())
    assert bool((torch.bincount(j, minlength=nq) == (cq.to(torch.int64) & 0xFFFFFFFF)).all())
    # sampled query points against the oracle (two-set join of all points with the sampled queries)
    qs = datagen.query_rows(w, 40, n=nq)
    sel = torch.zeros(nq, dtype=torch.bool, device="cuda")
    sel[torch.from_numpy(qs).cuda()] = True
    touch = sel[j]
    remap = torch.full((nq,), -1, dtype=torch.int64, device="cuda")
    remap[torch.from_numpy(qs).cuda()] = torch.arange(qs.size, device="cuda")
    sub = torch.stack([i[touch], remap[j[touch]]], 1).cpu().numpy().astype(np.uint32)
    subd = d2[:found][touch].cpu().numpy()
    P = orc.decode(X[:n])
    Q = orc.decode(np.ascontiguousarray(X[n:][qs]))
    op, od2 = orc.join_pairs(P, Q, eps)
    st = check_two_set(P, Q, eps, sub, subd, op, od2)
    print("  ", st, flush=True)
    assert st["oracle"] > 0


def test_full_size_split_join_against_oracle_rows(ej):
    """bench.py --mode split on workload 4's shape (2*10^6 x 384): FP32 points = the workload's FP16 values plus seeded
    noise below FP16 resolution; sampled rows against the FP64 join of the FP32 data."""
    w = 4
    spec = datagen.WORKLOADS[w]
    n, d = spec["n"], spec["d"]
    eps = stored_eps(w, 16)
    X = datagen.generate(w)
    rng = np.random.Generator(np.random.Philox(key=np.array([datagen.data_seed(w), 7], dtype=np.uint64)))
    X32 = X.view(np.float16).astype(np.float32)
    X32 += (rng.random(X32.shape, dtype=np.float32) - np.float32(0.5)) * np.float32(2.0 ** -12)
    Xd = torch.from_numpy(X32).cuda()
    cap = 40_000_000
    pairs, d2, npairs = ej.selfjoin_pairs_f32(Xd, eps, cap)
    torch.cuda.synchronize()
    assert ej.status() == 0
    found = int(npairs.cpu()[0])
    assert n < found <= cap
    i, j = gpu_pair_properties(pairs, found, n)
    q = datagen.query_rows(w, 48)
    sel = torch.zeros(n, dtype=torch.bool, device="cuda")
    sel[torch.from_numpy(q).cuda()] = True
    touch = sel[i] | sel[j]
    sub = torch.stack([i[touch], j[touch]], 1).cpu().numpy().astype(np.uint32)
    subd = d2[:found][touch].cpu().numpy()
    del pairs, d2, i, j, touch, Xd
    torch.cuda.empty_cache()
    P = X32.astype(np.float64)
    rs, nbr, nd2 = orc.rows_join(P, eps, q)
    st = parity.check_rows(P, eps, q, rs, nbr, nd2, sub, subd)
    print("  ", st, flush=True)
    assert st["d2_checked"] > 0
