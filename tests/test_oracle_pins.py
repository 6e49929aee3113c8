"""Pins for the CPU oracle: every check here compares the oracle with something that is not the
oracle -- other decoders, exact rational arithmetic, closed forms, counting arguments."""
import math
import struct
from fractions import Fraction

import numpy as np
import pytest

import datagen
from oracle import oracle as orc


# ------------------------------------------------------------------ fp16 decoding
def test_half_decode_exhaustive_against_two_decoders():
    bits = np.arange(65536, dtype=np.uint16)
    via_numpy = bits.view(np.float16).astype(np.float64)
    finite = np.isfinite(via_numpy)
    ours = np.array([orc.half_to_double(int(b)) for b in bits])
    via_struct = np.array([struct.unpack("<e", struct.pack("<H", int(b)))[0] for b in bits])
    assert np.array_equal(ours[finite], via_numpy[finite])
    assert np.array_equal(ours[finite], via_struct[finite])
    # signed zeros keep their sign, Inf/NaN are recognised
    assert math.copysign(1.0, orc.half_to_double(0x8000)) == -1.0
    assert np.array_equal(np.isnan(ours), np.isnan(via_numpy))
    assert np.array_equal(np.isinf(ours), np.isinf(via_numpy))


def test_decode_rejects_inf_nan_and_respects_ld():
    X = np.zeros((3, 8), dtype=np.uint16)
    X[:, :4] = np.float16(0.5).view(np.uint16)
    X[:, 4:] = 0x7C00  # padding columns hold Inf: must not be read when d = 4
    P = orc.decode(X, d=4)
    assert P.shape == (3, 4) and np.all(P == 0.5)
    with pytest.raises(ValueError):
        orc.decode(X)
    X[1, 2] = 0x7E00
    with pytest.raises(ValueError):
        orc.decode(X, d=4)


# ------------------------------------------------------------------ squared distances
def _frac_rows(X):
    return [[Fraction(struct.unpack("<e", struct.pack("<H", int(b)))[0]) for b in row] for row in X]


@pytest.mark.parametrize("n,d,seed", [(12, 7, 0), (9, 64, 1), (6, 200, 2)])
def test_dist2_against_exact_rational_arithmetic(n, d, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d)).astype(np.float16).view(np.uint16)  # signed, mixed magnitudes
    P = orc.decode(X)
    F = _frac_rows(X)
    full = orc.dist2_block(P, 0, n, 0, n)
    nrm = orc.norms(P)
    for i in range(n):
        exact_norm = sum(v * v for v in F[i])
        assert abs(Fraction(nrm[i]) - exact_norm) <= exact_norm * Fraction(d, 2**52)
        for j in range(n):
            exact = sum((a - b) ** 2 for a, b in zip(F[i], F[j]))
            got = orc.dist2(P, i, j)
            assert abs(Fraction(got) - exact) <= exact * Fraction(d, 2**52)
            assert got == full[i, j]
            if i == j:
                assert got == 0.0


def test_dist2_closed_forms_axis_aligned():
    d = 16
    vals = [0.5, 0.25, 1.0, 0.75, 3.0, 0.0009765625]
    rows = []
    for p, a in enumerate(vals):
        r = np.zeros(d, dtype=np.float16)
        r[p % 3] = a  # axes 0,1,2 : some share an axis, some do not
        rows.append(r)
    X = np.stack(rows).view(np.uint16)
    P = orc.decode(X)
    for i, a in enumerate(vals):
        for j, b in enumerate(vals):
            want = (a - b) ** 2 if (i % 3) == (j % 3) else a * a + b * b  # exact in double
            assert orc.dist2(P, i, j) == want


def test_dist2_grid_coordinates_integer_arithmetic():
    # coordinates are multiples of 2^-5 in [0,1]: D2 is an exact multiple of 2^-10
    rng = np.random.default_rng(3)
    q = rng.integers(0, 33, size=(40, 96))
    X = (q / 32.0).astype(np.float16).view(np.uint16)
    P = orc.decode(X)
    got = orc.dist2_block(P, 0, 40, 0, 40)
    want = ((q[:, None, :] - q[None, :, :]) ** 2).sum(-1)  # int64, exact
    assert np.array_equal(got * 1024.0, want.astype(np.float64))


def test_dist2_symmetry_and_orderings_bit_for_bit():
    X = datagen.generate(1, n=50)
    P = orc.decode(X)
    B = orc.dist2_block(P, 0, 50, 0, 50)
    assert np.array_equal(B, B.T)
    ap = orc.all_pairs_dist2(P)
    iu = np.triu_indices(50, 1)
    assert np.array_equal(ap, B[iu])  # (i, j>i) order, row-major
    sub = orc.dist2_block(P, 7, 5, 20, 11)
    assert np.array_equal(sub, B[7:12, 20:31])


def test_column_permutation_and_translation_invariance():
    # permuting coordinates only reorders the sum; translating by an fp16-exact shift keeps differences
    rng = np.random.default_rng(5)
    q = rng.integers(0, 17, size=(20, 32))
    X = (q / 32.0).astype(np.float16)
    P = orc.decode(X.view(np.uint16))
    perm = rng.permutation(32)
    P2 = orc.decode(np.ascontiguousarray(X[:, perm]).view(np.uint16))
    P3 = orc.decode((X + np.float16(0.25)).astype(np.float16).view(np.uint16))
    A = orc.dist2_block(P, 0, 20, 0, 20)
    assert np.array_equal(A, orc.dist2_block(P2, 0, 20, 0, 20))
    assert np.array_equal(A, orc.dist2_block(P3, 0, 20, 0, 20))


# ------------------------------------------------------------------ the join
def test_lattice_join_closed_form():
    n, d, h = 300, 8, 0.125
    X = datagen.lattice_points(n, d, h)
    P = orc.decode(X)
    for eps in [0.0, 0.1, 0.125, 0.3, 0.5, 1.0, 7.0625, 1000.0]:
        t = min(int(math.floor(float(np.float32(eps)) / h + 1e-12)), n - 1)
        want_pairs = sum(n - s for s in range(1, t + 1))
        counts, total = orc.selfjoin_count(P, eps)
        assert total == want_pairs
        idx = np.arange(n)
        assert np.array_equal(counts, np.minimum(t, idx) + np.minimum(t, n - 1 - idx))
        pairs, d2 = orc.selfjoin_pairs(P, eps)
        assert pairs.shape[0] == want_pairs + n
        # exact content: (i, j) with 0 <= j - i <= t, sorted
        want = [(i, j) for i in range(n) for j in range(i, min(n, i + t + 1))]
        assert pairs.tolist() == [list(p) for p in want]
        assert np.array_equal(d2, ((pairs[:, 1].astype(np.float64) - pairs[:, 0]) * h) ** 2)


def test_join_eps_zero_duplicates_and_eps_huge():
    X = datagen.generate(1, n=40)
    X[17] = X[3]
    X[29] = X[3]
    P = orc.decode(X)
    pairs, d2 = orc.selfjoin_pairs(P, 0.0)
    nonself = pairs[pairs[:, 0] != pairs[:, 1]].tolist()
    assert nonself == [[3, 17], [3, 29], [17, 29]]
    assert np.all(d2 == 0.0) and pairs.shape[0] == 43
    d = P.shape[1]
    pairs, _ = orc.selfjoin_pairs(P, math.sqrt(d) + 1e-3)  # coordinates lie in [0,1]
    assert pairs.shape[0] == 40 * 41 // 2
    counts, total = orc.selfjoin_count(P, math.sqrt(d) + 1e-3)
    assert total == 40 * 39 // 2 and np.all(counts == 39)


def test_threshold_is_inclusive():
    # two points at distance exactly 0.5 (fp32-exact epsilon): "<= eps" keeps the pair, a smaller eps drops it
    X = np.zeros((2, 4), dtype=np.float16)
    X[1, 2] = 0.5
    P = orc.decode(X.view(np.uint16))
    assert orc.selfjoin_count(P, 0.5)[1] == 1
    assert orc.selfjoin_count(P, np.nextafter(np.float32(0.5), np.float32(0)))[1] == 0


def test_counts_pairs_rows_agree_with_python_nested_loop():
    # second, differently written evaluation: pure-Python double loop over numpy float64 rows
    X = datagen.generate(2, n=64)
    P = orc.decode(X)
    n = 64
    eps = orc.select_eps_all_pairs(P, 6)
    e2 = float(np.float32(eps)) ** 2
    want = []
    for i in range(n):
        for j in range(i, n):
            s = 0.0
            for k in range(P.shape[1]):
                t = P[i, k] - P[j, k]
                s += t * t
            if s <= e2:
                want.append((i, j))
    pairs, d2 = orc.selfjoin_pairs(P, eps)
    assert [tuple(p) for p in pairs.tolist()] == want
    counts, total = orc.selfjoin_count(P, eps)
    ns = pairs[pairs[:, 0] != pairs[:, 1]]
    hist = np.bincount(ns[:, 0], minlength=n) + np.bincount(ns[:, 1], minlength=n)
    assert np.array_equal(counts, hist) and counts.sum() == 2 * total == 2 * len(ns)
    rows = np.array([0, 5, 63, 31], dtype=np.int64)
    rs, nbr, nd2 = orc.rows_join(P, eps, rows)
    for r, q in enumerate(rows):
        got = nbr[rs[r]:rs[r + 1]].tolist()
        exp = sorted([j for (i, j) in want if i == q and j != q] + [i for (i, j) in want if j == q and i != q])
        assert got == exp
        for j, v in zip(got, nd2[rs[r]:rs[r + 1]]):
            assert v == orc.dist2(P, q, j)


# ------------------------------------------------------------------ epsilon selection
def test_eps_selection_hits_the_requested_pair_count():
    X = datagen.generate(1, n=512)
    P = orc.decode(X)
    for S in (4, 32):
        eps = orc.select_eps_all_pairs(P, S)
        assert eps.dtype == np.float32
        _, total = orc.selfjoin_count(P, eps)
        assert total == S * 512 // 2  # no ties at the K-th distance for continuous data
    # sample rule: K = round(S/(n-1) * m(m-1)/2) pairs of the sample lie within eps
    Ps = P[:128]
    eps = orc.select_eps_sample(Ps, 64, n_full=1000)
    K = round(64 / 999 * (128 * 127 // 2))
    assert orc.selfjoin_count(Ps, eps)[1] == K


def test_uniform_data_moments_of_d2():
    # for independent U[0,1) coordinates E[(x-y)^2] = 1/6 and Var = 7/180 per coordinate
    X = datagen.generate(1, n=600)
    P = orc.decode(X)
    d = P.shape[1]
    v = orc.all_pairs_dist2(P)
    assert abs(v.mean() - d / 6) < 0.02 * d / 6
    assert abs(v.var() - 7 * d / 180) < 0.1 * 7 * d / 180


# ------------------------------------------------------------------ parity-rule helpers
def test_boundary_band_overlap_and_error_stats():
    eps = np.float32(2.0)
    d2 = np.array([4.0, (2.0 * 1.0009) ** 2, (2.0 * 1.0011) ** 2, (2.0 * 0.9991) ** 2, (2.0 * 0.9989) ** 2, 0.0])
    assert orc.boundary_band(d2, eps).tolist() == [True, True, False, True, False, False]
    a = np.array([[0, 0], [1, 1], [2, 2], [0, 1]], dtype=np.uint32)
    b = np.array([[0, 1], [0, 2]], dtype=np.uint32)
    # point 0: 1/2, point 1: 1/1, point 2: 0/1  (Eq. 3 of the paper, self excluded)
    assert orc.overlap_accuracy(3, a, b) == pytest.approx(0.5)
    assert orc.overlap_accuracy(3, a, a) == 1.0
    m, s = orc.distance_error_stats(np.array([4.0, 9.0]), np.array([1.0, 16.0]))
    assert m == pytest.approx(0.0) and s == pytest.approx(1.0)


# ------------------------------------------------------------------ two-set join
def test_two_set_join_against_python_loop_and_rational_arithmetic():
    rng = np.random.default_rng(21)
    XP = rng.standard_normal((23, 40)).astype(np.float16).view(np.uint16)
    XQ = rng.standard_normal((17, 40)).astype(np.float16).view(np.uint16)
    XQ[5] = XP[11]  # an exact duplicate across the sets: distance 0, must match for eps = 0
    P, Q = orc.decode(XP), orc.decode(XQ)
    FP, FQ = _frac_rows(XP), _frac_rows(XQ)
    B = orc.dist2_block2(P, Q, 0, 23, 0, 17)
    for i in range(23):
        for j in range(17):
            exact = sum((a - b) ** 2 for a, b in zip(FP[i], FQ[j]))
            assert abs(Fraction(B[i, j]) - exact) <= exact * Fraction(40, 2**52)
    assert B[11, 5] == 0.0
    pairs, d2 = orc.join_pairs(P, Q, 0.0)
    assert pairs.tolist() == [[11, 5]] and d2.tolist() == [0.0]
    eps = np.float32(np.sqrt(np.sort(B.ravel())[60]))
    e2 = float(eps) ** 2
    want = [(i, j) for i in range(23) for j in range(17) if B[i, j] <= e2]
    pairs, d2 = orc.join_pairs(P, Q, eps)
    assert [tuple(p) for p in pairs.tolist()] == want and np.array_equal(d2, B[pairs[:, 0], pairs[:, 1]])
    cp, cq, total = orc.join_count(P, Q, eps)
    assert total == len(want)
    assert np.array_equal(cp, np.bincount(pairs[:, 0], minlength=23)) and np.array_equal(cq, np.bincount(pairs[:, 1], minlength=17))
    assert np.array_equal(orc.dist2_block2(P, Q, 3, 4, 2, 9), B[3:7, 2:11])


def test_two_set_join_closed_form_shifted_lattices():
    # P: x = t*h, Q: x = u*h + h/2 on a line; |p_t - q_u| = |t - u - 1/2| h
    h, n_p, n_q = 0.25, 40, 33
    XP = datagen.lattice_points(n_p, 4, h)
    q = np.zeros((n_q, 4), dtype=np.float16)
    q[:, 0] = np.arange(n_q) * h + h / 2
    XQ = q.view(np.uint16)
    P, Q = orc.decode(XP), orc.decode(XQ)
    for eps in [0.1, 0.125, 0.3, 0.375, 1.0, 100.0]:
        e = float(np.float32(eps))
        want = [(t, u) for t in range(n_p) for u in range(n_q) if abs(t - u - 0.5) * h <= e]
        pairs, _ = orc.join_pairs(P, Q, eps)
        assert [tuple(p) for p in pairs.tolist()] == want
        assert orc.join_count(P, Q, eps)[2] == len(want)


def test_two_set_join_of_a_set_with_itself_is_the_full_self_join():
    X = datagen.generate(2, n=120)
    P = orc.decode(X)
    eps = orc.select_eps_all_pairs(P, 8)
    sp, _ = orc.selfjoin_pairs(P, eps)  # i <= j, self pairs included
    jp, _ = orc.join_pairs(P, P, eps)   # all ordered pairs
    ns = sp[sp[:, 0] != sp[:, 1]]
    want = sorted([tuple(p) for p in sp.tolist()] + [(j, i) for i, j in ns.tolist()])
    assert [tuple(p) for p in jp.tolist()] == want
    cp, cq, total = orc.join_count(P, P, eps)
    counts, t_self = orc.selfjoin_count(P, eps)
    assert total == 2 * t_self + 120 and np.array_equal(cp, counts + 1) and np.array_equal(cq, cp)


# ------------------------------------------------------------------ ingestion
def _f32(v):
    return struct.unpack("<f", struct.pack("<f", v))[0]  # Python double -> nearest-even FP32


def _f16_bits(v):
    try:
        return struct.unpack("<H", struct.pack("<e", v))[0]  # struct rounds to nearest even
    except OverflowError:
        return 0x7C00 if v > 0 else 0xFC00


def test_convert_f32_rounds_to_nearest_even_like_an_independent_encoder():
    rng = np.random.default_rng(31)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32) * np.float32(3.0),
                        np.array([0.0, -0.0, 1.0, 65504.0, 65519.9, 65520.0, 1e-8, 5.96e-8, 2.98e-8, 2.0**-24 * 1.5,
                                  1.0009765625, 1.00048828125, 1.00146484375], dtype=np.float32)])
    scale = np.float32(0.7)
    got = orc.convert_f32(x.reshape(1, -1), scale)[0, :x.size]
    # products of two FP32 numbers are exact in double, so each stage below rounds exactly once
    want = [_f16_bits(_f32(float(v) * float(scale))) for v in x.tolist()]
    assert got.tolist() == want
    # with a shift: x - c is exact in double for these magnitudes, then rounded to FP32, then scaled
    c = (rng.standard_normal(x.size) * 2).astype(np.float32)
    X2 = np.stack([x, x[::-1]])
    got = orc.convert_f32(X2, scale, center=c)[:, :x.size]
    for r in range(2):
        want = [_f16_bits(_f32(_f32(float(v) - float(cc)) * float(scale))) for v, cc in zip(X2[r].tolist(), c.tolist())]
        assert got[r].tolist() == want
    # ties go to even: 1 + 2^-11 (half-way between 1 and 1 + 2^-10) -> 1 ; 1 + 3*2^-11 -> 1 + 2^-9
    t = orc.convert_f32(np.array([[1.00048828125, 1.00146484375]], dtype=np.float32), 1.0)[0, :2]
    assert t.tolist() == [0x3C00, 0x3C02]
    # padding columns are zero, the layout is (n, roundup(d, 64))
    p = orc.convert_f32(np.ones((3, 70), dtype=np.float32))
    assert p.shape == (3, 128) and np.all(p[:, 70:] == 0) and np.all(p[:, :70] == 0x3C00)
