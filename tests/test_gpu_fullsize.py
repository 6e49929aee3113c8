"""Parity at the full sizes of the five workloads, in the launch configuration bench.py times.

Workloads 1 and 2 are joined in full by the oracle; workloads 3-5 are checked on 512 seeded query rows whose
exact FP64 neighbour lists are held against the neighbours the GPU pair list has for them, plus properties
of the whole GPU output that hold at any size (tests/fullsize.py).  All five are held to the STRICT rule:
mismatches only inside the relative 1e-3 band around epsilon, squared distances within a relative 1e-3.
"""
import numpy as np
import pytest
import torch

import datagen
from oracle import oracle as orc
from tests import fullsize, parity
from tests.fullsize import gpu_pair_properties, stored_eps

pytestmark = pytest.mark.gpu
ROWS = 512


@pytest.fixture(scope="module")
def ej():
    import paper_2508_21230_amd as pkg
    e = pkg.EJoin(0)
    yield e
    e.close()


@pytest.mark.parametrize("w,S,rows", [(1, 32, None), (2, 64, None), (3, 16, ROWS), (4, 16, ROWS), (4, 128, ROWS), (4, 1024, ROWS), (5, 64, ROWS)])
def test_full_size_pairs_against_the_oracle_strict_rule(ej, w, S, rows):
    st = fullsize.check_workload(ej, w, S, rows)
    assert st["d2_checked"] > 0
    assert st.get("floor_used", 0) == 0
    # Mismatches exist only among the boundary pairs (the strict rule above); of those at most one in seven falls on
    # the other side.  What that does to the overlap accuracy of Eq. 3 depends on how much of the distance distribution
    # epsilon cuts through: where under 3 % of the neighbours are boundary pairs (workloads 1, 2, 5, workload 4 at S = 1024)
    # it stays above the paper's own worst value (Table "accuracy": 0.99946); workload 3 (d = 960: distances concentrate,
    # a tenth of all neighbours lie within 1e-3 of epsilon) reads 0.992, workload 4 at S = 16 / 128 reads 0.9986 / 0.9989.
    checked = st.get("neighbours_oracle", st.get("pairs_oracle"))
    assert st["boundary_mismatch_rate"] <= 0.15
    assert st["overlap_accuracy"] >= (0.9994 if st["boundary_pairs"] <= 0.03 * checked else 0.99)
    # no measurable bias (Section 4.5): the mean distance error is a small fraction of its spread
    assert abs(st["dist_err_mean"]) <= 0.25 * st["dist_err_std"] + 1e-7


def test_scale_12m_points_against_oracle_rows(ej):
    """Not one of the task's configurations: 12 M points at d = 64 (1.1e9 tiles, exactly as many slices per tile as
    the copy pipeline runs ahead) as a test of scale; ordinary rule, 32 query rows."""
    fullsize.oracle_side.cache_clear()
    w, S, rows = 6, 64, 32
    spec = datagen.WORKLOADS[w]
    n = spec["n"]
    eps = stored_eps(w, S)
    X = datagen.generate(w)
    Xd = torch.from_numpy(X.view(np.int16)).cuda()
    capacity = int(n * (S / 2 + 1) * 1.6) + (1 << 20)
    pairs, d2, npairs = ej.selfjoin_pairs(Xd, eps, capacity)
    torch.cuda.synchronize()
    assert ej.status() == 0
    found = int(npairs.cpu()[0])
    assert found <= capacity
    i, j = gpu_pair_properties(pairs, found, n)
    q = datagen.query_rows(w, rows)
    sel = torch.zeros(n, dtype=torch.bool, device="cuda")
    sel[torch.from_numpy(q).cuda()] = True
    touch = sel[i] | sel[j]
    sub = torch.stack([i[touch], j[touch]], 1).cpu().numpy().astype(np.uint32)
    subd = d2[:found][touch].cpu().numpy()
    del pairs, d2, i, j, touch, Xd
    torch.cuda.empty_cache()
    P = orc.decode(X)
    rs, nbr, nd2 = orc.rows_join(P, eps, q)
    st = parity.check_rows(P, eps, q, rs, nbr, nd2, sub, subd)
    print("  ", st, flush=True)
    assert st["d2_checked"] > 0


def test_full_size_two_set_join_against_oracle_queries(ej):
    """bench.py --mode join at its full size: the 10^6 points of workload 3 against 10^5 query points; 40 sampled
    query points are joined exactly by the oracle, the whole output is checked for range, duplicates and counts."""
    from tests.test_gpu_twoset import check_two_set
    fullsize.oracle_side.cache_clear()
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
