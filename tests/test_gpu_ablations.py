"""The ablation builds of the join kernel (build.ABLATIONS: one design element taken out each) compute the same
result as the full kernel: every variant is held to the parity rule against the CPU oracle, through the C ABI, on a
case of several tiles per workgroup-free grid and one with ragged edges.  (bench_ablation.py, which times them,
compares pair counts only.)  The variants are built by `python -m paper_2508_21230_amd.build --ablations`, which
__graft_entry__.build() runs; a variant that is not built is skipped, never faked."""
import os

import numpy as np
import pytest
import torch

import datagen
from oracle import oracle as orc
from paper_2508_21230_amd import build
from tests import parity

pytestmark = pytest.mark.gpu

CASES = [(2, 3001, 40), (4, 1300, 24), (1, 700, 12)]  # (workload shape, n, neighbours per point epsilon is chosen for)


@pytest.fixture(scope="module")
def oracle_results():
    out = []
    for w, n, S in CASES:
        X = datagen.generate(w, n=n)
        P = orc.decode(X)
        eps = float(orc.select_eps_all_pairs(P, S))
        pairs, d2 = orc.selfjoin_pairs(P, eps)
        out.append((X, P, eps, pairs, d2))
    return out


@pytest.mark.parametrize("name", sorted(build.ABLATIONS))
def test_ablation_variant_passes_the_parity_rule(name, oracle_results):
    import paper_2508_21230_amd as pkg
    path = os.path.join(build.ABLATION_DIR, f"libejoin_{name}.so")
    if not os.path.exists(path):
        pytest.skip(f"{path} is not built (python -m paper_2508_21230_amd.build --ablations)")
    sources = [build.SRC, os.path.join(os.path.dirname(build.SRC), "tile_cursor.h"), os.path.join(os.path.dirname(build.SRC), "panel_layout.h")]
    if os.path.getmtime(path) < max(os.path.getmtime(f) for f in sources):
        pytest.skip(f"{path} is older than the kernel source: rebuild the variants")
    ej = pkg.EJoin(0, lib_path=path)
    try:
        for X, P, eps, opairs, od2 in oracle_results:
            Xd = torch.from_numpy(X.view(np.int16)).cuda()
            pairs, d2, npairs = ej.selfjoin_pairs(Xd, eps, capacity=opairs.shape[0] + 4096)
            counts, total = ej.selfjoin_count(Xd, eps)
            torch.cuda.synchronize()
            assert ej.status() == 0
            hp, hd2, found = parity.to_host_pairs(pairs, d2, npairs)
            st = parity.check_pair_sets(P, eps, hp, hd2, opairs, od2)
            assert int(total.cpu()[0]) == found - P.shape[0]
            ns = hp[hp[:, 0] != hp[:, 1]].astype(np.int64)
            hist = np.bincount(ns[:, 0], minlength=P.shape[0]) + np.bincount(ns[:, 1], minlength=P.shape[0])
            assert np.array_equal(hist, counts.cpu().numpy().view(np.uint32).astype(np.int64))
            assert st["overlap_accuracy"] > 0.999
    finally:
        ej.close()
