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
