"""GPU parity tests: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import math

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


def pad(X, ld):
    out = np.zeros((X.shape[0], ld), dtype=np.uint16)
    out[:, :X.shape[1]] = X
    return out


def run_pairs(ej, Xd, eps, capacity, d=None, with_dist2=True):
    p, d2, npairs = ej.selfjoin_pairs(Xd, eps, capacity, d=d, with_dist2=with_dist2)
    torch.cuda.synchronize()
    return parity.to_host_pairs(p, d2, npairs)


def small_case(workload, n, S):
    X = datagen.generate(workload, n=n)
    P = orc.decode(X)
    eps = orc.select_eps_all_pairs(P, S)
    return X, P, eps


# ------------------------------------------------------------------ Step 1: norms
@pytest.mark.parametrize("workload,n", [(1, 1000), (3, 777), (4, 300)])
def test_norms_against_oracle(ej, workload, n):
    print(f"norms workload={workload} n={n}", flush=True)
    X = datagen.generate(workload, n=n)
    P = orc.decode(X)
    s = ej.norms(dev(X)).cpu().numpy().astype(np.float64)
    want = orc.norms(P)
    d = X.shape[1]
    # one RNE rounding per MFMA step (32-wide; at most d/16 of them) on a running sum <= s: |err| <= (d/16 + 1) * 2^-24 * s
    assert np.all(np.abs(s - want) <= (d / 16 + 1) * 2.0**-24 * want)


# ------------------------------------------------------------------ Steps 2-3: dense tile
@pytest.mark.parametrize("workload,n,i0,j0,rows,cols", [(1, 600, 0, 0, 600, 600), (3, 500, 37, 250, 301, 199), (4, 400, 390, 5, 10, 33)])
def test_dist2_tile_against_oracle(ej, workload, n, i0, j0, rows, cols):
    print(f"dist2_tile workload={workload} n={n} block=({i0},{j0},{rows},{cols})", flush=True)
    X = datagen.generate(workload, n=n)
    # a copy of a row elsewhere in the block: its distance to the original is computed like any other (only the
    # diagonal itself is written as 0 by definition) and must be exactly 0 -- the norms are the Gram diagonal bit for bit
    ri, cj = i0 + rows // 3, j0 + (2 * cols) // 3
    if ri != cj:
        X[cj] = X[ri]
    P = orc.decode(X)
    got = ej.dist2_tile(dev(X), i0, j0, rows, cols).cpu().numpy().astype(np.float64)
    want = orc.dist2_block(P, i0, rows, j0, cols)
    if ri != cj:
        assert got[ri - i0, cj - j0] == 0.0
    s = orc.norms(P)
    tol = parity.value_tolerance(want, s[i0:i0 + rows, None] + s[None, j0:j0 + cols], s.max())
    assert np.all(np.abs(got - want) <= tol)
    if i0 == j0 and rows == cols:
        assert np.array_equal(got, got.T)


# ------------------------------------------------------------------ the join, element by element
@pytest.mark.parametrize("workload,n,S", [(1, 4096, 32), (2, 5000, 64), (3, 3000, 16), (4, 2500, 128), (5, 3333, 64)])
def test_selfjoin_pairs_against_oracle(ej, workload, n, S):
    print(f"selfjoin_pairs workload={workload} n={n} S={S}", flush=True)
    X, P, eps = small_case(workload, n, S)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    pairs, d2, found = run_pairs(ej, dev(X), eps, capacity=ora_pairs.shape[0] + 4096)
    assert found == pairs.shape[0]
    st = parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)
    print("  ", st, flush=True)
    assert st["overlap_accuracy"] >= 0.9994  # the paper's worst overlap accuracy against FP64 (Table "accuracy")
    assert abs(st["dist_err_mean"]) < 1e-4


def test_join_dist2_is_bit_identical_to_dense_tile(ej):
    X, P, eps = small_case(2, 1500, 40)
    Xd = dev(X)
    pairs, d2, found = run_pairs(ej, Xd, eps, capacity=200000)
    dense = ej.dist2_tile(Xd, 0, 0, 1500, 1500).cpu().numpy()
    assert np.array_equal(dense[pairs[:, 0], pairs[:, 1]], d2)
    # and the filter is exactly "d2 <= fl(eps*eps)" on those values
    e2 = np.float32(eps) * np.float32(eps)
    iu = np.triu_indices(1500, 1)
    assert int((dense[iu] <= e2).sum()) + 1500 == found


def test_count_mode_equals_histogram_of_pair_mode(ej):
    X, P, eps = small_case(5, 4000, 50)
    Xd = dev(X)
    pairs, _, found = run_pairs(ej, Xd, eps, capacity=400000, with_dist2=False)
    counts, total = ej.selfjoin_count(Xd, eps)
    torch.cuda.synchronize()
    counts = counts.cpu().numpy().view(np.uint32)
    ns = pairs[pairs[:, 0] != pairs[:, 1]]
    hist = np.bincount(ns[:, 0], minlength=4000) + np.bincount(ns[:, 1], minlength=4000)
    assert np.array_equal(counts, hist)
    assert int(total.cpu()[0]) == ns.shape[0] == found - 4000
    # against the oracle: counts may differ only through boundary pairs
    oc, ot = orc.selfjoin_count(P, eps)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    st = parity.check_pair_sets(P, eps, pairs, None, ora_pairs, ora_d2)
    assert abs(int(ot) - ns.shape[0]) <= st["only_gpu"] + st["only_oracle"]


def test_run_to_run_same_set(ej):
    X, P, eps = small_case(2, 3000, 64)
    Xd = dev(X)
    a, da, _ = run_pairs(ej, Xd, eps, capacity=300000)
    b, db, _ = run_pairs(ej, Xd, eps, capacity=300000)
    ka, kb = orc.pair_keys(a), orc.pair_keys(b)
    oa, ob = np.argsort(ka), np.argsort(kb)
    assert np.array_equal(ka[oa], kb[ob]) and np.array_equal(da[oa], db[ob])


# ------------------------------------------------------------------ edge cases
@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 255, 256, 257, 1000])
@pytest.mark.parametrize("d", [64, 192])
def test_edge_sizes(ej, n, d):
    print(f"edge n={n} d={d}", flush=True)
    rng = np.random.default_rng(n * 1000 + d)
    X = rng.random((n, d), dtype=np.float32).astype(np.float16).view(np.uint16)
    P = orc.decode(X)
    eps = np.float32(math.sqrt(d / 6.0) * 0.9) if n > 1 else np.float32(1.0)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    pairs, d2, found = run_pairs(ej, dev(X), eps, capacity=n * (n + 1) // 2 + 8)
    assert found == pairs.shape[0]
    parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)


@pytest.mark.parametrize("n,d", [(6500, 64), (7000, 40), (6200, 128), (5900, 192), (12000, 64), (11000, 24), (12000, 128), (11000, 100)])
def test_more_tiles_than_workgroups_at_small_d(ej, n, d):
    """Every workgroup walks several tiles (351 .. 406 tiles on 256 workgroups; 946 and 1128 in the last two cases,
    four to five per workgroup).  At d <= 64 a tile has two slices and the copy pipeline runs three ahead: the copy
    cursor works on the tile after the next one while the current one is still being computed.  At 96 < d <= 128 a tile
    has as many slices as the LDS ring has stages, and a row panel stays in the LDS across the consecutive tiles of a
    workgroup that share it (the last two cases: four to five tiles per workgroup, three of four with the row of the
    tile before)."""
    print(f"multi-tile n={n} d={d}", flush=True)
    rng = np.random.default_rng(n + d)
    X = rng.random((n, d), dtype=np.float32).astype(np.float16).view(np.uint16)
    P = orc.decode(X)
    eps = orc.select_eps_sample(P[np.sort(rng.choice(n, size=1500, replace=False))], 8, n)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    ld = (d + 63) // 64 * 64
    pairs, d2, found = run_pairs(ej, dev(pad(X, ld)), eps, capacity=ora_pairs.shape[0] * 2 + 1024, d=d)
    assert found == pairs.shape[0]
    parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)
    # count mode walks the same schedule
    counts, total = ej.selfjoin_count(dev(pad(X, ld)), eps, d=d)
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == found - n


@pytest.mark.parametrize("n,d", [(700, 2048), (300, 4096), (900, 1), (900, 33)])
def test_extreme_dimensionalities(ej, n, d):
    print(f"extreme d: n={n} d={d}", flush=True)
    rng = np.random.default_rng(17 * d + n)
    X = rng.random((n, d), dtype=np.float32).astype(np.float16).view(np.uint16)
    P = orc.decode(X)
    eps = orc.select_eps_all_pairs(P, 12)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    ld = (d + 63) // 64 * 64
    pairs, d2, found = run_pairs(ej, dev(pad(X, ld)), eps, capacity=ora_pairs.shape[0] * 2 + 1024, d=d)
    assert found == pairs.shape[0]
    parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)


@pytest.mark.parametrize("kind", ["small", "mixed", "tiny_among_large"])
def test_small_and_mixed_norms(ej, kind):
    """The norm term of the expansion is carried as three FP16 pieces scaled to the largest norm of the data:
    data of small norm, and points of very different norms in one set, must meet the same parity bar."""
    rng = np.random.default_rng({"small": 1, "mixed": 2, "tiny_among_large": 3}[kind])
    n, d = 1200, 128
    X32 = rng.random((n, d), dtype=np.float32)
    if kind == "small":
        X32 *= np.float32(0.01)                       # s ~ 4e-3
    elif kind == "mixed":
        X32 *= (10.0 ** rng.uniform(-2.5, 0.5, size=(n, 1))).astype(np.float32)   # s from ~4e-4 to ~4e2
    else:
        X32[: n // 2] *= np.float32(2.0 ** -11)       # s ~ 1e-5 next to s ~ 40: ratio above 2^16
        X32[n // 2:] *= np.float32(1.0)
    X = X32.astype(np.float16).view(np.uint16)
    X[7] = X[3]                                        # an exact duplicate among the first (small-norm) points
    P = orc.decode(X)
    eps = orc.select_eps_all_pairs(P, 10)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    pairs, d2, found = run_pairs(ej, dev(X), eps, capacity=ora_pairs.shape[0] * 2 + 1024)
    parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)
    # epsilon = 0: every self pair, with distance 0, whatever the norms; the duplicate too where the norm term is exact
    pairs0, d20, found0 = run_pairs(ej, dev(X), 0.0, capacity=4 * n)
    keys = set(map(tuple, pairs0.tolist()))
    assert all((i, i) in keys for i in range(n))
    assert np.all(d20[pairs0[:, 0] == pairs0[:, 1]] == 0.0)
    if kind != "tiny_among_large":
        assert (3, 7) in keys and found0 == n + 1
    D = ej.dist2_tile(dev(X), 0, 0, 64, 64).cpu().numpy()
    if kind != "tiny_among_large":
        assert D[3, 7] == 0.0 and D[7, 3] == 0.0  # the duplicate, off the diagonal: computed, not written as 0


def test_unpadded_d_with_zero_columns(ej):
    # d = 100 stored with ld = 128 and zero padding (the paper pads d to a multiple of 64 with zeros)
    rng = np.random.default_rng(5)
    X = rng.random((700, 100), dtype=np.float32).astype(np.float16).view(np.uint16)
    P = orc.decode(X)
    eps = orc.select_eps_all_pairs(P, 20)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    pairs, d2, found = run_pairs(ej, dev(pad(X, 128)), eps, capacity=40000, d=100)
    parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)


def test_eps_zero_and_duplicates(ej):
    X = datagen.generate(1, n=700)
    X[300] = X[5]
    X[699] = X[5]
    X[256] = X[255]
    P = orc.decode(X)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, 0.0)
    pairs, d2, found = run_pairs(ej, dev(X), 0.0, capacity=2000)
    # duplicates are at distance exactly 0 on the GPU too (norms are the Gram diagonal), so the sets are equal
    k = np.argsort(orc.pair_keys(pairs))
    assert np.array_equal(pairs[k], ora_pairs) and np.all(d2 == 0.0)


def test_all_identical_points_and_eps_huge(ej):
    n = 300
    X = np.tile(datagen.generate(1, n=1), (n, 1))
    pairs, d2, found = run_pairs(ej, dev(X), 0.0, capacity=n * (n + 1) // 2)
    assert found == n * (n + 1) // 2 == pairs.shape[0] and np.all(d2 == 0.0)
    assert np.unique(orc.pair_keys(pairs)).size == found
    X = datagen.generate(1, n=n)
    pairs, d2, found = run_pairs(ej, dev(X), 1000.0, capacity=n * (n + 1) // 2)
    assert found == n * (n + 1) // 2 and np.unique(orc.pair_keys(pairs)).size == found
    counts, total = ej.selfjoin_count(dev(X), 1000.0)
    assert int(total.cpu()[0]) == n * (n - 1) // 2 and np.all(counts.cpu().numpy() == n - 1)


def test_capacity_overflow_reports_found_and_writes_capacity(ej):
    X, P, eps = small_case(1, 1024, 32)
    Xd = dev(X)
    full, _, found = run_pairs(ej, Xd, eps, capacity=100000)
    cap = 1000
    p = torch.full((cap + 64, 2), -1, dtype=torch.int32, device="cuda")
    _, _, npairs = ej.selfjoin_pairs(Xd, eps, cap, pairs=p, with_dist2=False)
    torch.cuda.synchronize()
    assert int(npairs.cpu()[0]) == found > cap
    h = p.cpu().numpy()
    assert np.all(h[cap:] == -1), "wrote past capacity"
    got = h[:cap].view(np.uint32)
    assert np.all(np.isin(orc.pair_keys(got), orc.pair_keys(full)))
    assert np.unique(orc.pair_keys(got)).size == cap


def test_invalid_arguments_are_rejected(ej):
    import paper_2508_21230_amd as pkg
    X = torch.zeros((10, 128), dtype=torch.float16, device="cuda")
    with pytest.raises(pkg.EJoinError):
        ej.selfjoin_pairs(X[:, :100], 1.0, 10)          # ld = 128 but d = 100 is fine; d > ld is not
        ej.selfjoin_pairs(X, 1.0, 10, d=200)
    with pytest.raises(pkg.EJoinError):
        ej.selfjoin_pairs(X, -1.0, 10)
    Y = torch.zeros((10, 96), dtype=torch.float16, device="cuda")
    with pytest.raises(pkg.EJoinError):
        ej.norms(Y)                                      # ld not a multiple of 64
    Z = torch.zeros(10 * 128 + 8, dtype=torch.float16, device="cuda")[8:].view(10, 128)
    with pytest.raises(pkg.EJoinError):
        ej.norms(Z)                                      # base not 128-byte aligned


# ------------------------------------------------------------------ data range
def test_large_norms_use_the_scaled_split(ej):
    # Sift-like data: integer coordinates 0..218 in d = 128 (the paper's Sift10M has epsilon ~ 122-152,
    # data-set table); norms ~ 1e6 exceed the FP16 range of -s/2, so the augmentation rows are scaled.
    rng = np.random.default_rng(11)
    n, d = 1500, 128
    centres = rng.integers(0, 219, size=(12, d))
    X = np.clip(centres[rng.integers(0, 12, size=n)] + rng.normal(0, 8, size=(n, d)).round(), 0, 218).astype(np.float16).view(np.uint16)
    P = orc.decode(X)
    assert orc.norms(P).max() > 3e5
    eps = orc.select_eps_all_pairs(P, 30)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    pairs, d2, found = run_pairs(ej, dev(X), eps, capacity=ora_pairs.shape[0] + 4096)
    assert ej.status() == 0
    st = parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)
    print("  ", st, flush=True)
    dense = ej.dist2_tile(dev(X), 0, 0, n, n).cpu().numpy()
    assert np.array_equal(dense[pairs[:, 0], pairs[:, 1]], d2)


def test_status_reports_out_of_range_and_non_finite_input(ej):
    n, d = 600, 64
    X = datagen.generate(1, n=n)[:, :d].copy()
    Xd = dev(X)
    # fine
    _, _, npairs = ej.selfjoin_pairs(Xd, 1.0, 1000)
    assert ej.status() == 0
    # norms >= 2^31: 64 coordinates of 60000 -> s = 2.3e11
    big = np.full((n, d), np.float16(60000.0)).view(np.uint16)
    p, d2, npairs = ej.selfjoin_pairs(dev(big), 1.0, 1000)
    assert ej.status() == 1 and int(npairs.cpu()[0]) == 0
    counts, total = ej.selfjoin_count(dev(big), 1.0)
    assert ej.status() == 1 and int(total.cpu()[0]) == 0 and int(counts.cpu().abs().sum()) == 0
    # Inf in the input
    bad = X.copy()
    bad[17, 3] = 0x7C00
    p, d2, npairs = ej.selfjoin_pairs(dev(bad), 1.0, 1000)
    assert ej.status() == 2 and int(npairs.cpu()[0]) == 0
    # and the context recovers
    _, _, npairs = ej.selfjoin_pairs(Xd, 1.0, 1000)
    assert ej.status() == 0 and int(npairs.cpu()[0]) >= n


def test_count_mode_on_dense_output(ej):
    # whole clusters within epsilon: every 32 x 32 block of most tiles holds hits
    X = datagen.generate(4, n=6000)
    P = orc.decode(X)
    eps = orc.select_eps_all_pairs(P, 900)
    Xd = dev(X)
    oc, ot = orc.selfjoin_count(P, eps)
    counts, total = ej.selfjoin_count(Xd, eps)
    pairs, _, found = run_pairs(ej, Xd, eps, capacity=int(ot * 1.1) + 8000, with_dist2=False)
    counts = counts.cpu().numpy().view(np.uint32)
    ns = pairs[pairs[:, 0] != pairs[:, 1]]
    hist = np.bincount(ns[:, 0], minlength=6000) + np.bincount(ns[:, 1], minlength=6000)
    assert np.array_equal(counts, hist) and int(total.cpu()[0]) == ns.shape[0]
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    st = parity.check_pair_sets(P, eps, pairs, None, ora_pairs, ora_d2)
    assert abs(int(ot) - ns.shape[0]) <= st["only_gpu"] + st["only_oracle"]


def test_convert_f32_matches_the_oracle_bit_for_bit(ej):
    rng = np.random.default_rng(41)
    for n, d, scale, centred in [(1000, 100, 1.0, False), (333, 960, 0.01, True), (5, 64, 7.5, True), (2, 1, 1.0, False)]:
        X32 = (rng.standard_normal((n, d)) * 40).astype(np.float32)
        X32.flat[::97] = 1e6  # overflows FP16 unless scaled down -> Inf on both sides
        c = (rng.standard_normal(d) * 10).astype(np.float32) if centred else None
        got = ej.convert_f32(torch.from_numpy(X32).cuda(), scale, None if c is None else torch.from_numpy(c).cuda())
        want = orc.convert_f32(X32, scale, c)
        got = got.cpu().numpy().view(np.uint16)
        assert got.shape == want.shape and np.array_equal(got, want)
    # the converted array feeds the join directly
    X32 = rng.random((600, 100), dtype=np.float32)
    Xd = ej.convert_f32(torch.from_numpy(X32).cuda())
    P = orc.decode(orc.convert_f32(X32), d=100)
    eps = orc.select_eps_all_pairs(P, 10)
    ora_pairs, ora_d2 = orc.selfjoin_pairs(P, eps)
    pairs, d2, found = run_pairs(ej, Xd, eps, capacity=20000, d=100)
    parity.check_pair_sets(P, eps, pairs, d2, ora_pairs, ora_d2)


def test_centring_and_scaling_recover_accuracy_on_offset_data(ej):
    """Data far from the origin converts badly to FP16 (Section 5): shifted and scaled ingestion brings the
    result set back to that of the FP64 join on the original FP32 data (overlap accuracy, Eq. 3)."""
    rng = np.random.default_rng(43)
    n, d = 1500, 64
    X32 = (100.0 + rng.random((n, d))).astype(np.float32)  # spacing of FP16 near 100 is 1/16
    truth = X32.astype(np.float64)
    eps = orc.select_eps_all_pairs(truth, 32)
    want = orc.selfjoin_pairs(truth, eps)[0]
    Xg = torch.from_numpy(X32).cuda()
    c = torch.from_numpy(X32.mean(axis=0).astype(np.float32)).cuda()
    acc = {}
    for name, scale, centre in [("raw", 1.0, None), ("centred", 1.0, c), ("centred_scaled", 4.0, c)]:
        Xd = ej.convert_f32(Xg, scale, centre)
        pairs, _, found = run_pairs(ej, Xd, eps * scale, capacity=400000, d=d)
        assert found <= 400000
        acc[name] = orc.overlap_accuracy(n, want, pairs)
    assert acc["raw"] < 0.9
    assert acc["centred"] > 0.99 and acc["centred_scaled"] >= acc["centred"] - 1e-3


def test_join_calls_can_be_captured_in_a_hip_graph_and_replayed(ej):
    """With the workspace reserved a join enqueues kernels only (no allocation, no memset node), so a caller
    may capture it; every replay, on new data in the same buffers, must equal the eager result."""
    rng = np.random.default_rng(61)
    n, d = 3000, 128
    ej.reserve(n, d)
    Xd = torch.empty((n, d), dtype=torch.int16, device="cuda")
    cap = 200000
    pairs = torch.empty((cap, 2), dtype=torch.int32, device="cuda")
    d2 = torch.empty(cap, dtype=torch.float32, device="cuda")
    npairs = torch.zeros(1, dtype=torch.int64, device="cuda")
    counts = torch.empty(n, dtype=torch.int32, device="cuda")
    total = torch.zeros(1, dtype=torch.int64, device="cuda")
    eps = 3.9
    datasets = [rng.random((n, d), dtype=np.float32).astype(np.float16).view(np.int16) for _ in range(3)]
    Xd.copy_(torch.from_numpy(datasets[0]))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on the capture stream, as torch asks
        ej.selfjoin_pairs(Xd, eps, cap, pairs=pairs, dist2=d2, n_pairs=npairs)
        ej.selfjoin_count(Xd, eps, counts=counts, total=total)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ej.selfjoin_pairs(Xd, eps, cap, pairs=pairs, dist2=d2, n_pairs=npairs)
        ej.selfjoin_count(Xd, eps, counts=counts, total=total)
    for rep in range(4):
        X = datasets[rep % 3]
        Xd.copy_(torch.from_numpy(X))
        g.replay()
        torch.cuda.synchronize()
        gp, gd2, found = parity.to_host_pairs(pairs, d2, npairs)
        gc, gt = counts.cpu().numpy().copy(), int(total.cpu()[0])
        # eager run on the same data (own buffers), with host synchronisation in between
        ep, ed2, en = ej.selfjoin_pairs(Xd, eps, cap)
        ec, et = ej.selfjoin_count(Xd, eps)
        torch.cuda.synchronize()
        hp, hd2, hfound = parity.to_host_pairs(ep, ed2, en)
        assert found == hfound and found > n and gt == int(et.cpu()[0]) == found - n
        oa, ob = np.argsort(orc.pair_keys(gp)), np.argsort(orc.pair_keys(hp))
        assert np.array_equal(gp[oa], hp[ob]) and np.array_equal(gd2[oa], hd2[ob])
        assert np.array_equal(gc, ec.cpu().numpy())


def test_contexts_and_prepared_sets_release_their_device_memory():
    import paper_2508_21230_amd as pkg
    X = torch.zeros((5000, 128), dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for _ in range(20):
        e = pkg.EJoin(0)
        e.reserve(200_000, 256)            # ~100 MB of workspace
        s = e.prepare(X)
        counts, total = e.selfjoin_count(X, 0.5)
        torch.cuda.synchronize()
        s.close()
        e.close()
    del counts, total
    torch.cuda.synchronize()
    free1 = torch.cuda.mem_get_info()[0]
    assert free0 - free1 < 64 << 20, f"device memory not returned: {free0 - free1} bytes"


@pytest.mark.parametrize("batches", [1, 3, 32])
def test_batched_return_to_host_gives_the_pairs_of_the_plain_join(ej, batches):
    """ejoin_selfjoin_pairs_to_host: the join cut into launches by rows of super-blocks, each batch copied to pinned host
    memory while the next computes -- same pair set and squared distances as ejoin_selfjoin_pairs, also when the
    buffer overflows (exactly `capacity` pairs returned, the count still complete)."""
    n = 21_000  # 83 tiles per side: six rows of super-blocks
    X = datagen.generate(2, n=n)
    Xd = torch.from_numpy(X.view(np.int16)).cuda()
    eps = 0.78
    want_pairs, want_d2, want_n = ej.selfjoin_pairs(Xd, eps, capacity=4_000_000)
    torch.cuda.synchronize()
    wp, wd, found = parity.to_host_pairs(want_pairs, want_d2, want_n)
    assert n < found < 4_000_000
    cap = found + 100
    pairs = torch.empty((cap, 2), dtype=torch.int32, device="cuda")
    d2 = torch.empty(cap, dtype=torch.float32, device="cuda")
    hp = torch.empty((cap, 2), dtype=torch.int32).pin_memory()
    hd = torch.empty(cap, dtype=torch.float32).pin_memory()
    got = ej.selfjoin_pairs_to_host(Xd, eps, batches, pairs, d2, hp, hd)
    assert got == found
    assert ej.status() == 0
    gp = hp[:got].numpy().view(np.uint32)
    ko, kg = orc.pair_keys(wp), orc.pair_keys(gp)
    oo, og = np.argsort(ko), np.argsort(kg)
    assert np.array_equal(ko[oo], kg[og])
    assert np.array_equal(wd[oo].view(np.uint32), hd[:got].numpy()[og].view(np.uint32))
    # overflow: a buffer of half the size
    small = found // 2
    got2 = ej.selfjoin_pairs_to_host(Xd, eps, batches, pairs[:small], d2[:small], hp[:small], hd[:small])
    assert got2 == found
    sub = orc.pair_keys(hp[:small].numpy().view(np.uint32))
    assert np.unique(sub).size == small and np.isin(sub, ko).all()


def test_status_waits_for_the_stream_of_the_call(ej):
    """ejoin_status must order against the stream the join ran on, also a non-blocking side stream that the null
    stream does not wait for: a join over data with an Inf, queued behind other work on such a stream, then status()
    with no device synchronisation in between."""
    n, d = 30_000, 128
    good = torch.from_numpy(datagen.generate(2, n=n).view(np.int16)).cuda()
    bad = good.clone()
    bad[7, 3] = 0x7C00  # +Inf
    ej.selfjoin_count(good, 0.5)
    torch.cuda.synchronize()
    assert ej.status() == 0
    side = torch.cuda.Stream()
    a = torch.randn(4096, 4096, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(20):  # tens of milliseconds of work ahead of the join
            a = a @ a * 1e-3
        counts, total = ej.selfjoin_count(bad, 0.5)
        st = ej.status()
    assert st == 2
    torch.cuda.synchronize()
    assert int(total.cpu()[0]) == 0
