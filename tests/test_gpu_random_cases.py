"""Seeded random parity cases: sizes, dimensionalities, value scales, selectivities and modes drawn at random,
each compared with the CPU oracle under the rule of tests/parity.py.  The fixed cases elsewhere pin the known
corners; these walk the space between them (several tiles per workgroup at small d, ragged everything)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from tests import parity
from tests.test_gpu_twoset import check_two_set

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ej():
    import paper_2508_21230_amd as pkg
    e = pkg.EJoin(0)
    yield e
    e.close()


def dev(X):
    return torch.from_numpy(X.view(np.int16)).cuda()


def draw_points(rng, n, d, ld):
    kind = rng.integers(0, 3)
    scale = np.float32(10.0 ** rng.uniform(-2.0, 1.0))
    if kind == 0:
        x = rng.random((n, d), dtype=np.float32)
    elif kind == 1:  # clustered
        k = int(rng.integers(1, 20))
        x = rng.random((k, d), dtype=np.float32)[rng.integers(0, k, size=n)] + np.float32(0.03) * rng.standard_normal((n, d)).astype(np.float32)
    else:            # signed, heavy-tailed
        x = rng.standard_t(4, size=(n, d)).astype(np.float32) * np.float32(0.3)
    out = np.zeros((n, ld), dtype=np.uint16)
    out[:, :d] = (x * scale).astype(np.float16).view(np.uint16)
    return out


@pytest.mark.parametrize("seed", range(24))
def test_random_self_join(ej, seed):
    rng = np.random.default_rng(50_000 + seed)
    d = int(rng.choice([1, 7, 31, 32, 33, 64, 65, 100, 128, 200, 257, 320]))
    n = int(rng.integers(1, 7500 if d <= 64 else 2600))
    ld = (d + 63) // 64 * 64 + 64 * int(rng.integers(0, 2))
    X = draw_points(rng, n, d, ld)
    P = orc.decode(X[:, :d])
    S = min(float(rng.choice([0.5, 4, 30])), 0.8 * (n - 1))  # mean neighbours per point, fewer than there are points
    eps = orc.select_eps_all_pairs(P, S) if n >= 3 and S * n / 2 >= 1 else np.float32(0.0)
    print(f"random self-join seed={seed} n={n} d={d} ld={ld} S={S} eps={eps}", flush=True)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    pairs, d2, npairs = ej.selfjoin_pairs(dev(X), float(eps), ora_pairs.shape[0] * 2 + 1024, d=d)
    torch.cuda.synchronize()
    assert ej.status() == 0
    gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
    assert found == gp.shape[0]
    parity.check_pair_sets(P, eps, gp, gd2, ora_pairs, ora_d2)
    counts, total = ej.selfjoin_count(dev(X), float(eps), d=d)
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == found - n
    off = gp[gp[:, 0] != gp[:, 1]]
    hist = np.bincount(off[:, 0], minlength=n) + np.bincount(off[:, 1], minlength=n)
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), hist)


@pytest.mark.parametrize("seed", range(12))
def test_random_two_set_join(ej, seed):
    rng = np.random.default_rng(60_000 + seed)
    d = int(rng.choice([3, 64, 96, 128, 130, 256]))
    n_p = int(rng.integers(1, 5000 if d <= 64 else 2500))
    n_q = int(rng.integers(1, 5000 if d <= 64 else 2500))
    ld = (d + 63) // 64 * 64
    both = draw_points(rng, n_p + n_q, d, ld)
    XP, XQ = np.ascontiguousarray(both[:n_p]), np.ascontiguousarray(both[n_p:])
    P, Q = orc.decode(XP[:, :d]), orc.decode(XQ[:, :d])
    B = orc.dist2_block2(P, Q, 0, min(n_p, 1500), 0, min(n_q, 1500)).ravel()
    eps = orc.eps_for_pair_rank(B, max(1, min(B.size - 1, int(B.size * 10.0 ** rng.uniform(-4, -2)))))
    print(f"random two-set seed={seed} np={n_p} nq={n_q} d={d} eps={eps}", flush=True)
    op, od2 = orc.join_pairs(P, Q, eps)
    pairs, d2, npairs = ej.join_pairs(dev(XP), dev(XQ), float(eps), capacity=op.shape[0] * 2 + 1024, d=d)
    torch.cuda.synchronize()
    assert ej.status() == 0
    gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
    assert found == gp.shape[0]
    check_two_set(P, Q, eps, gp, gd2, op, od2)


@pytest.mark.parametrize("seed", range(8))
def test_random_multi_tile_dense_output_and_overflow(ej, seed):
    """5000 .. 9500 points (every workgroup walks several tiles), up to hundreds of neighbours per point, and in a
    third of the cases a result buffer half the size needed: the count keeps running, what was written is valid."""
    rng = np.random.default_rng(70_000 + seed)
    d = int(rng.choice([16, 64, 65, 128, 192]))
    n = int(rng.integers(5000, 9500))
    ld = (d + 63) // 64 * 64
    X = draw_points(rng, n, d, ld)
    P = orc.decode(X[:, :d])
    S = float(rng.choice([2, 40, 300]))
    eps = orc.select_eps_sample(P[np.sort(rng.choice(n, size=1500, replace=False))], S, n)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    small_cap = bool(rng.integers(0, 3) == 0)
    cap = (ora_pairs.shape[0] // 2) if small_cap else ora_pairs.shape[0] * 2 + 1024
    print(f"random multi-tile seed={seed} n={n} d={d} S={S} eps={eps} pairs={ora_pairs.shape[0]} cap={cap}", flush=True)
    pairs, d2, npairs = ej.selfjoin_pairs(dev(X), float(eps), cap, d=d)
    torch.cuda.synchronize()
    assert ej.status() == 0
    gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
    if small_cap:
        assert found > cap and gp.shape[0] == cap
        kg = orc.pair_keys(gp)
        assert np.unique(kg).size == kg.size
        extra = gp[~np.isin(kg, orc.pair_keys(ora_pairs))]
        if extra.size:
            s = orc.norms(P)
            d2x = np.array([orc.dist2(P, int(i), int(j)) for i, j in extra])
            assert parity.in_band(d2x, eps, s[extra[:, 0]] + s[extra[:, 1]], s.max()).all()
    else:
        assert found == gp.shape[0]
        parity.check_pair_sets(P, eps, gp, gd2, ora_pairs, ora_d2)
    counts, total = ej.selfjoin_count(dev(X), float(eps), d=d)
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == found - n
