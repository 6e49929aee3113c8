"""GPU parity of the two-set join (points P x query points Q) against the CPU oracle."""
import numpy as np
import pytest
import torch

import datagen
from oracle import oracle as orc
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ej():
    import paper_2508_21230_amd as pkg
    e = pkg.EJoin(0)
    yield e
    e.close()


def dev(X):
    return torch.from_numpy(X.view(np.int16)).cuda()


def check_two_set(P, Q, eps, gp, gd2, op, od2):
    """Parity rule of tests/parity.py for a two-set result (no self pairs, i indexes P, j indexes Q)."""
    assert gp.size == 0 or (gp[:, 0].max() < P.shape[0] and gp[:, 1].max() < Q.shape[0])
    kg = orc.pair_keys(gp)
    order = np.argsort(kg)
    kgs = kg[order]
    assert np.all(kgs[1:] != kgs[:-1]), "duplicate pairs"
    ko = orc.pair_keys(op)
    cg, co = np.isin(kgs, ko, assume_unique=True), np.isin(ko, kgs, assume_unique=True)
    sp, sq = orc.norms(P), orc.norms(Q)
    s_max = max(sp.max(), sq.max())
    oo = op[~co]
    assert parity.in_band(od2[~co], eps, sp[oo[:, 0]] + sq[oo[:, 1]], s_max).all(), "missed a pair outside the boundary band"
    only_g = kgs[~cg]
    if only_g.size:
        gi = (only_g >> np.uint64(32)).astype(np.int64)
        gj = (only_g & np.uint64(0xFFFFFFFF)).astype(np.int64)
        d2x = np.array([orc.dist2_block2(P, Q, int(i), 1, int(j), 1)[0, 0] for i, j in zip(gi, gj)])
        assert parity.in_band(d2x, eps, sp[gi] + sq[gj], s_max).all(), "extra pair outside the boundary band"
    g = gd2[order][cg].astype(np.float64)
    o = od2[co]
    pp = op[co]
    tol = parity.value_tolerance(o, sp[pp[:, 0]] + sq[pp[:, 1]], s_max)
    assert (np.abs(g - o) <= tol).all()
    return dict(gpu=len(kg), oracle=len(ko), only_gpu=int(only_g.size), only_oracle=int((~co).sum()))


@pytest.mark.parametrize("w,n_p,n_q,S", [(2, 3000, 1700, 30), (3, 700, 2100, 12), (4, 257, 255, 40), (5, 1, 900, 5), (1, 4096, 256, 16)])
def test_two_set_pairs_against_oracle(ej, w, n_p, n_q, S):
    print(f"two-set w={w} np={n_p} nq={n_q}", flush=True)
    X = datagen.generate(w, n=n_p + n_q)
    XP, XQ = np.ascontiguousarray(X[:n_p]), np.ascontiguousarray(X[n_p:])
    P, Q = orc.decode(XP), orc.decode(XQ)
    B = orc.dist2_block2(P, Q, 0, n_p, 0, n_q).ravel()
    K = min(int(S * n_p), B.size - 1)
    eps = orc.eps_for_pair_rank(B, max(K, 1))
    op, od2 = orc.join_pairs(P, Q, eps)
    pairs, d2, npairs = ej.join_pairs(dev(XP), dev(XQ), float(eps), capacity=op.shape[0] + 4096)
    torch.cuda.synchronize()
    assert ej.status() == 0
    gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
    assert found == gp.shape[0]
    st = check_two_set(P, Q, eps, gp, gd2, op, od2)
    print("  ", st, flush=True)
    # counts agree with the pair list
    cp, cq, total = ej.join_count(dev(XP), dev(XQ), float(eps))
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == found
    assert np.array_equal(cp.cpu().numpy().view(np.uint32), np.bincount(gp[:, 0], minlength=n_p))
    assert np.array_equal(cq.cpu().numpy().view(np.uint32), np.bincount(gp[:, 1], minlength=n_q))
    cp2, none, total2 = ej.join_count(dev(XP), dev(XQ), float(eps), want_counts_q=False)
    assert none is None and int(total2.cpu()[0]) == found and torch.equal(cp2, cp)


@pytest.mark.parametrize("d,n_p,n_q", [(64, 4200, 4400), (128, 4200, 4400), (64, 9000, 7100), (128, 8000, 9100)])
def test_two_set_more_tiles_than_workgroups(ej, d, n_p, n_q):
    # 17 x 18 = 306 tiles on 256 workgroups, or 36 x 28 = 1008 (about four per workgroup); at d <= 64 a tile has fewer
    # slices than the copies run ahead, and the copy cursor is two tiles ahead of the tile being computed
    rng = np.random.default_rng(900 + d)
    XP = rng.random((n_p, d), dtype=np.float32).astype(np.float16).view(np.uint16)
    XQ = rng.random((n_q, d), dtype=np.float32).astype(np.float16).view(np.uint16)
    P, Q = orc.decode(XP), orc.decode(XQ)
    eps = orc.eps_for_pair_rank(orc.dist2_block2(P, Q, 0, 1200, 0, 1200).ravel(), 3000)
    op, od2 = orc.join_pairs(P, Q, eps)
    pairs, d2, npairs = ej.join_pairs(dev(XP), dev(XQ), float(eps), capacity=op.shape[0] * 2 + 4096)
    torch.cuda.synchronize()
    gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
    assert found == gp.shape[0]
    print("  ", check_two_set(P, Q, eps, gp, gd2, op, od2), flush=True)
    # count mode walks the same schedule
    cp, cq, total = ej.join_count(dev(XP), dev(XQ), float(eps))
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == found
    assert np.array_equal(cp.cpu().numpy().view(np.uint32), np.bincount(gp[:, 0], minlength=n_p))
    assert np.array_equal(cq.cpu().numpy().view(np.uint32), np.bincount(gp[:, 1], minlength=n_q))


def test_two_set_join_of_a_set_with_itself_matches_the_self_join(ej):
    X = datagen.generate(2, n=2000)
    P = orc.decode(X)
    eps = orc.select_eps_all_pairs(P, 25)
    Xd = dev(X)
    sp, sd2, snp = ej.selfjoin_pairs(Xd, float(eps), 200000)
    jp, jd2, jnp = ej.join_pairs(Xd, Xd, float(eps), 400000)
    torch.cuda.synchronize()
    s_pairs, s_d2, s_found = parity.to_host_pairs(sp, sd2, snp)
    j_pairs, j_d2, j_found = parity.to_host_pairs(jp, jd2, jnp)
    ns = s_pairs[:, 0] != s_pairs[:, 1]
    assert j_found == 2 * int(ns.sum()) + 2000
    # same arithmetic: (i, j) of the two-set join carries the bits the self-join reports for {i, j}
    both = np.concatenate([s_pairs, s_pairs[ns][:, ::-1]])
    both_d2 = np.concatenate([s_d2, s_d2[ns]])
    ka, kb = orc.pair_keys(both), orc.pair_keys(j_pairs)
    oa, ob = np.argsort(ka), np.argsort(kb)
    assert np.array_equal(ka[oa], kb[ob]) and np.array_equal(both_d2[oa], j_d2[ob])


def test_two_set_duplicates_across_sets_and_eps_zero(ej):
    XP = datagen.generate(1, n=300)
    XQ = datagen.generate(5, n=500)[:, :128].copy()
    XQ[7] = XP[100]
    XQ[499] = XP[299]
    pairs, d2, npairs = ej.join_pairs(dev(XP), dev(XQ), 0.0, 100)
    torch.cuda.synchronize()
    gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
    assert sorted(map(tuple, gp.tolist())) == [(100, 7), (299, 499)] and np.all(gd2 == 0.0)


def test_two_set_rejects_mismatched_inputs(ej):
    import paper_2508_21230_amd as pkg
    A = torch.zeros((10, 128), dtype=torch.float16, device="cuda")
    B = torch.zeros((10, 192), dtype=torch.float16, device="cuda")
    with pytest.raises(pkg.EJoinError):
        ej.join_pairs(A, B, 1.0, 10)


def test_prepared_set_gives_the_results_of_the_plain_two_set_join(ej):
    """Three query batches against one prepared set, the second with norms far above the set's (the norm
    terms of the set are rescaled per call), then the first again: each bit-identical to ejoin_join_pairs."""
    rng = np.random.default_rng(77)
    d = 100
    XP = np.zeros((3000, 128), dtype=np.uint16)
    XP[:, :d] = rng.random((3000, d), dtype=np.float32).astype(np.float16).view(np.uint16)
    batches = []
    for n_q, scale in [(700, 1.0), (1300, 30.0), (257, 0.05)]:
        XQ = np.zeros((n_q, 128), dtype=np.uint16)
        XQ[:, :d] = (rng.random((n_q, d), dtype=np.float32) * np.float32(scale)).astype(np.float16).view(np.uint16)
        batches.append(XQ)
    Pd = dev(XP)
    pset = ej.prepare(Pd, d=d)
    P = orc.decode(XP[:, :d])
    for k in (0, 1, 2, 0):
        XQ = batches[k]
        Q = orc.decode(XQ[:, :d])
        eps = orc.eps_for_pair_rank(orc.dist2_block2(P, Q, 0, 3000, 0, XQ.shape[0]).ravel(), 2000)
        a = ej.join_pairs(Pd, dev(XQ), float(eps), 50000, d=d)
        torch.cuda.synchronize()
        ap, ad2, af = parity.to_host_pairs(*a)
        b = pset.join_pairs(dev(XQ), float(eps), 50000)
        torch.cuda.synchronize()
        assert ej.status() == 0
        bp, bd2, bf = parity.to_host_pairs(*b)
        assert af == bf
        oa, ob = np.argsort(orc.pair_keys(ap)), np.argsort(orc.pair_keys(bp))
        assert np.array_equal(ap[oa], bp[ob]) and np.array_equal(ad2[oa], bd2[ob])
        # and against the oracle
        op, od2 = orc.join_pairs(P, Q, eps)
        check_two_set(P, Q, eps, bp, bd2, op, od2)
        cp, cq, total = pset.join_count(dev(XQ), float(eps))
        torch.cuda.synchronize()
        assert int(total.cpu()[0]) == bf
        assert np.array_equal(cp.cpu().numpy().view(np.uint32), np.bincount(bp[:, 0], minlength=3000))
        assert np.array_equal(cq.cpu().numpy().view(np.uint32), np.bincount(bp[:, 1], minlength=XQ.shape[0]))
    pset.close()
    # a set belongs to its context, and d comes from the set
    import paper_2508_21230_amd as pkg
    other = pkg.EJoin(0)
    s2 = other.prepare(Pd, d=d)
    with pytest.raises(pkg.EJoinError):
        ej._check(ej._lib.ejoin_set_join_pairs(ej._h, s2._h, Pd.data_ptr(), 10, 128, 1.0, Pd.data_ptr(), None, 1, Pd.data_ptr(), None), ej._h)
    s2.close()
    other.close()
