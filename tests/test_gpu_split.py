"""GPU parity of the split-FP16 self-join of FP32 rows against the CPU oracle evaluated on the FP32 data in FP64."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ej():
    import paper_2508_21230_amd as pkg
    e = pkg.EJoin(0)
    yield e
    e.close()


def run_f32(ej, X32, eps, capacity):
    pairs, d2, npairs = ej.selfjoin_pairs_f32(torch.from_numpy(X32).cuda(), float(eps), capacity)
    torch.cuda.synchronize()
    assert ej.status() == 0
    return parity.to_host_pairs(pairs, d2, npairs)


def data(kind, n, d, seed):
    rng = np.random.default_rng(seed)
    if kind == "uniform":
        return rng.random((n, d), dtype=np.float32)
    if kind == "offset":      # far from the origin: FP16 spacing near 10 is 2^-7
        return (np.float32(10.0) + rng.random((n, d), dtype=np.float32)).astype(np.float32)
    if kind == "clustered":
        c = rng.random((12, d), dtype=np.float32)
        return (c[rng.integers(0, 12, size=n)] + np.float32(0.03) * rng.standard_normal((n, d)).astype(np.float32)).astype(np.float32)
    raise ValueError(kind)


@pytest.mark.parametrize("kind,n,d,ld_extra", [("uniform", 1500, 100, 0), ("offset", 1300, 64, 5), ("clustered", 2100, 257, 0),
                                               ("uniform", 1, 8, 0), ("uniform", 700, 1, 3), ("clustered", 6300, 48, 0)])
def test_split_join_matches_fp64_on_the_fp32_data(ej, kind, n, d, ld_extra):
    print(f"split {kind} n={n} d={d}", flush=True)
    X = data(kind, n, d, seed=n + d)
    if ld_extra:
        buf = np.full((n, d + ld_extra), np.float32(123.0))  # columns beyond d must be ignored
        buf[:, :d] = X
        Xarg = buf[:, :d]
    else:
        Xarg = X
    P = X.astype(np.float64)
    eps = orc.select_eps_all_pairs(P, 8) if n >= 3 else np.float32(0.5)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    Xd = torch.from_numpy(np.ascontiguousarray(buf) if ld_extra else X).cuda()
    if ld_extra:
        Xd = Xd[:, :d]
    pairs, d2, npairs = ej.selfjoin_pairs_f32(Xd, float(eps), ora_pairs.shape[0] * 2 + 1024)
    torch.cuda.synchronize()
    assert ej.status() == 0
    gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
    assert found == gp.shape[0]
    st = parity.check_pair_sets(P, eps, gp, gd2, ora_pairs, ora_d2)
    print("  ", st, flush=True)
    counts, total = ej.selfjoin_count_f32(Xd, float(eps))
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == found - n
    off = gp[gp[:, 0] != gp[:, 1]]
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), np.bincount(off[:, 0], minlength=n) + np.bincount(off[:, 1], minlength=n))


def test_split_join_is_more_accurate_than_the_fp16_join_where_conversion_hurts(ej):
    """Points in [10, 11]^64: converted to FP16 their coordinates move by up to 2^-8, a quarter of the typical
    neighbour distance; the split join sees 22 bits of every coordinate."""
    n, d = 2000, 64
    X = data("offset", n, d, seed=5)
    P = X.astype(np.float64)
    eps = orc.select_eps_all_pairs(P, 16)
    truth = orc.selfjoin_pairs(P, eps)[0]
    gp, gd2, found = run_f32(ej, X, eps, 400000)
    acc_split = orc.overlap_accuracy(n, truth, gp)
    X16 = ej.convert_f32(torch.from_numpy(X).cuda())
    p16, d16, n16 = ej.selfjoin_pairs(X16, float(eps), 400000, d=d)
    torch.cuda.synchronize()
    g16, _, _ = parity.to_host_pairs(p16, d16, n16)
    acc_fp16 = orc.overlap_accuracy(n, truth, g16)
    print(f"  overlap accuracy: split {acc_split:.5f}, fp16 {acc_fp16:.5f}", flush=True)
    assert acc_split > 0.995 and acc_split > acc_fp16 + 0.01  # what is left is the FP32 accumulation at s ~ 7000
    # squared distances: the split join's error is that of the FP32 accumulation, not of the conversion
    common = np.isin(orc.pair_keys(gp), orc.pair_keys(truth))
    o = {int(k): v for k, v in zip(orc.pair_keys(truth), orc.selfjoin_pairs(P, eps)[1])}
    err = np.array([abs(float(v) - o[int(k)]) for k, v in zip(orc.pair_keys(gp)[common], gd2[common])])
    s_max = (P ** 2).sum(axis=1).max()
    assert err.max() <= 2e-6 * s_max


def test_split_join_duplicates_and_self_pairs(ej):
    rng = np.random.default_rng(9)
    X = rng.standard_normal((900, 70)).astype(np.float32)
    X[100] = X[5]
    X[899] = X[5]
    gp, gd2, found = run_f32(ej, X, 0.0, 4000)
    keys = set(map(tuple, gp.tolist()))
    assert found == 900 + 3 and {(5, 100), (5, 899), (100, 899)} <= keys
    assert np.all(gd2 == 0.0)


def test_split_join_rejects_bad_arguments_and_reports_out_of_range_data(ej):
    import paper_2508_21230_amd as pkg
    X = torch.zeros((10, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(pkg.EJoinError):
        ej.selfjoin_pairs_f32(X, -1.0, 100)
    with pytest.raises(pkg.EJoinError):
        ej.selfjoin_pairs_f32(X.to(torch.float64), 1.0, 100)
    big = torch.full((10, 8), 1.0e5, dtype=torch.float32, device="cuda")  # beyond FP16's largest number
    pairs, d2, npairs = ej.selfjoin_pairs_f32(big, 1.0, 100)
    torch.cuda.synchronize()
    assert ej.status() == 2 and int(npairs.cpu()[0]) == 0
