"""Python face of the CPU oracle for the epsilon self-join.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg.  The product path (the HIP library and its binding) never imports it, and
this module never imports the product.

The arithmetic lives in ejoin_oracle.c (plain C, FP64, difference form of Eq. 1 of the paper);
this file marshals numpy arrays to it and adds the small numpy-only steps that are part of
the oracle's definition: epsilon selection from a distance quantile, the boundary-band
classification used by the parity rule, the overlap accuracy of Eq. 3 and the distance-error
statistic of Section 4.5.

Pins (tests/test_oracle_*.py): exhaustive fp16 decode against two independent decoders;
exact rational arithmetic (fractions.Fraction) on small inputs; closed forms (identical
points, axis-aligned points, a 1-D lattice with a closed-form pair count, eps = 0, eps >= sqrt(d));
symmetry; counts == histogram of the pair list; U[0,1) moments of D2; the two-set join against the
self-join of the stacked sets and against exact rational arithmetic; the FP32 -> FP16 ingestion
(convert_f32) against an independent round-to-nearest-even encoder.  No function here is unpinned.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ejoin_oracle.c")
_LIB = os.path.join(_HERE, "libejoin_oracle.so")

# AVX2-level code so that a library built on one x86-64 host runs on another; contraction off
# so that the arithmetic is exactly the one written in the C file.
CFLAGS = ["-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (a few seconds)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        p = C.c_void_p
        lib.orc_half_to_double.restype = C.c_double
        lib.orc_half_to_double.argtypes = [C.c_uint16]
        lib.orc_decode.restype = C.c_int
        lib.orc_decode.argtypes = [p, C.c_int64, C.c_int32, C.c_int64, p]
        lib.orc_num_threads.restype = C.c_int
        lib.orc_dist2.restype = C.c_double
        lib.orc_dist2.argtypes = [p, C.c_int32, C.c_int64, C.c_int64]
        lib.orc_norms.restype = None
        lib.orc_norms.argtypes = [p, C.c_int64, C.c_int32, p]
        lib.orc_dist2_block.restype = None
        lib.orc_dist2_block.argtypes = [p, C.c_int32, C.c_int64, C.c_int32, C.c_int64, C.c_int32, p]
        lib.orc_all_pairs_dist2.restype = None
        lib.orc_all_pairs_dist2.argtypes = [p, C.c_int64, C.c_int32, p]
        lib.orc_selfjoin_count.restype = C.c_int64
        lib.orc_selfjoin_count.argtypes = [p, C.c_int64, C.c_int32, C.c_double, p]
        lib.orc_selfjoin_pairs.restype = C.c_int64
        lib.orc_selfjoin_pairs.argtypes = [p, C.c_int64, C.c_int32, C.c_double, p, p, C.c_int64, p]
        lib.orc_rows_join.restype = C.c_int64
        lib.orc_rows_join.argtypes = [p, C.c_int64, C.c_int32, C.c_double, p, C.c_int64, p, p, p]
        lib.orc_join_count.restype = C.c_int64
        lib.orc_join_count.argtypes = [p, C.c_int64, p, C.c_int64, C.c_int32, C.c_double, p, p]
        lib.orc_join_pairs.restype = C.c_int64
        lib.orc_join_pairs.argtypes = [p, C.c_int64, p, C.c_int64, C.c_int32, C.c_double, p, p, C.c_int64, p]
        lib.orc_dist2_block2.restype = None
        lib.orc_dist2_block2.argtypes = [p, p, C.c_int32, C.c_int64, C.c_int32, C.c_int64, C.c_int32, p]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(_L().orc_num_threads())


def half_to_double(bits: int) -> float:
    return float(_L().orc_half_to_double(int(bits) & 0xFFFF))


def decode(X: np.ndarray, d: int | None = None) -> np.ndarray:
    """fp16 bit patterns (n, ld) uint16 -> dense (n, d) float64.  Raises on Inf/NaN."""
    assert X.dtype == np.uint16 and X.ndim == 2
    n, ld = X.shape
    d = ld if d is None else d
    Xc = np.ascontiguousarray(X)
    P = np.empty((n, d), dtype=np.float64)
    if _L().orc_decode(_ptr(Xc), n, d, ld, _ptr(P)) != 0:
        raise ValueError("input holds Inf or NaN")
    return P


def convert_f32(X32: np.ndarray, scale=1.0, center=None, ld16: int | None = None) -> np.ndarray:
    """Ingestion as its definition states it: fp16_rne(fl32(scale * fl32(x - center))), zero padded; uint16 bits."""
    X32 = np.asarray(X32, dtype=np.float32)
    n, d = X32.shape
    ld16 = (d + 63) // 64 * 64 if ld16 is None else ld16
    out = np.zeros((n, ld16), dtype=np.float16)
    t = X32 if center is None else X32 - np.asarray(center, dtype=np.float32)[None, :]
    with np.errstate(over="ignore"):
        out[:, :d] = (t * np.float32(scale)).astype(np.float16)
    return out.view(np.uint16)


def eps2_of(eps) -> float:
    """Threshold on squared distances: the FP32 epsilon squared in FP64."""
    e = float(np.float32(eps))
    return e * e


def dist2(P: np.ndarray, i: int, j: int) -> float:
    return float(_L().orc_dist2(_ptr(P), P.shape[1], int(i), int(j)))


def norms(P: np.ndarray) -> np.ndarray:
    s = np.empty(P.shape[0], dtype=np.float64)
    _L().orc_norms(_ptr(P), P.shape[0], P.shape[1], _ptr(s))
    return s


def dist2_block(P: np.ndarray, i0: int, rows: int, j0: int, cols: int) -> np.ndarray:
    n = P.shape[0]
    assert 0 <= i0 and i0 + rows <= n and 0 <= j0 and j0 + cols <= n
    out = np.empty((rows, cols), dtype=np.float64)
    _L().orc_dist2_block(_ptr(P), P.shape[1], i0, rows, j0, cols, _ptr(out))
    return out


def all_pairs_dist2(P: np.ndarray) -> np.ndarray:
    m = P.shape[0]
    out = np.empty(m * (m - 1) // 2, dtype=np.float64)
    _L().orc_all_pairs_dist2(_ptr(P), m, P.shape[1], _ptr(out))
    return out


def selfjoin_count(P: np.ndarray, eps) -> tuple[np.ndarray, int]:
    """(counts[i] = neighbours of i excluding i, number of pairs i<j)."""
    counts = np.empty(P.shape[0], dtype=np.uint32)
    total = _L().orc_selfjoin_count(_ptr(P), P.shape[0], P.shape[1], eps2_of(eps), _ptr(counts))
    return counts, int(total)


def selfjoin_pairs(P: np.ndarray, eps) -> tuple[np.ndarray, np.ndarray]:
    """(pairs (m, 2) uint32 sorted by (i, j) with i <= j, self pairs included; D2 (m,) float64)."""
    n, d = P.shape
    row_start = np.empty(n + 1, dtype=np.int64)
    e2 = eps2_of(eps)
    found = _L().orc_selfjoin_pairs(_ptr(P), n, d, e2, None, None, 0, _ptr(row_start))
    pairs = np.empty((found, 2), dtype=np.uint32)
    d2 = np.empty(found, dtype=np.float64)
    again = _L().orc_selfjoin_pairs(_ptr(P), n, d, e2, _ptr(pairs), _ptr(d2), found, _ptr(row_start))
    assert again == found
    return pairs, d2


def rows_join(P: np.ndarray, eps, rows: np.ndarray) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Neighbour lists of the query rows: (row_start (R+1,), neighbours uint32, D2 float64)."""
    n, d = P.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < n)
    R = rows.size
    row_start = np.zeros(R + 1, dtype=np.int64)
    e2 = eps2_of(eps)
    total = _L().orc_rows_join(_ptr(P), n, d, e2, _ptr(rows), R, _ptr(row_start), None, None)
    nbr = np.empty(total, dtype=np.uint32)
    d2 = np.empty(total, dtype=np.float64)
    _L().orc_rows_join(_ptr(P), n, d, e2, _ptr(rows), R, _ptr(row_start), _ptr(nbr), _ptr(d2))
    return row_start, nbr, d2


def join_count(P: np.ndarray, Q: np.ndarray, eps) -> tuple[np.ndarray, np.ndarray, int]:
    """Two-set join: (counts_p[i] = matches of p_i in Q, counts_q[j] = matches of q_j in P, total)."""
    assert P.shape[1] == Q.shape[1]
    cp = np.empty(P.shape[0], dtype=np.uint32)
    cq = np.empty(Q.shape[0], dtype=np.uint32)
    total = _L().orc_join_count(_ptr(P), P.shape[0], _ptr(Q), Q.shape[0], P.shape[1], eps2_of(eps), _ptr(cp), _ptr(cq))
    return cp, cq, int(total)


def join_pairs(P: np.ndarray, Q: np.ndarray, eps) -> tuple[np.ndarray, np.ndarray]:
    """Two-set join: (pairs (m, 2) uint32 sorted by (i, j), i indexes P and j indexes Q; D2 (m,))."""
    assert P.shape[1] == Q.shape[1]
    n_p, d = P.shape
    row_start = np.empty(n_p + 1, dtype=np.int64)
    e2 = eps2_of(eps)
    found = _L().orc_join_pairs(_ptr(P), n_p, _ptr(Q), Q.shape[0], d, e2, None, None, 0, _ptr(row_start))
    pairs = np.empty((found, 2), dtype=np.uint32)
    d2 = np.empty(found, dtype=np.float64)
    again = _L().orc_join_pairs(_ptr(P), n_p, _ptr(Q), Q.shape[0], d, e2, _ptr(pairs), _ptr(d2), found, _ptr(row_start))
    assert again == found
    return pairs, d2


def dist2_block2(P: np.ndarray, Q: np.ndarray, i0: int, rows: int, j0: int, cols: int) -> np.ndarray:
    assert 0 <= i0 and i0 + rows <= P.shape[0] and 0 <= j0 and j0 + cols <= Q.shape[0]
    out = np.empty((rows, cols), dtype=np.float64)
    _L().orc_dist2_block2(_ptr(P), _ptr(Q), P.shape[1], i0, rows, j0, cols, _ptr(out))
    return out


# ---------------------------------------------------------------------------------------------
# epsilon selection (part of the workload definition; the paper picks epsilon per data set so
# that the selectivity S = (|R| - |D|) / |D| hits a target, Section 4.1.3)
# ---------------------------------------------------------------------------------------------

def eps_for_pair_rank(D2_all: np.ndarray, K: int) -> np.float32:
    """Epsilon (FP32) lying between the K-th and (K+1)-th smallest pair distance, K >= 1."""
    m = D2_all.size
    K = int(K)
    assert 1 <= K < m
    part = np.partition(D2_all, [K - 1, K])
    lo, hi = np.sqrt(part[K - 1]), np.sqrt(part[K])
    return np.float32(0.5 * (lo + hi))


def select_eps_all_pairs(P: np.ndarray, S: float) -> np.float32:
    """Epsilon giving mean S neighbours/point over the whole set: K = S*n/2 unordered pairs."""
    n = P.shape[0]
    return eps_for_pair_rank(all_pairs_dist2(P), int(round(S * n / 2)))


def select_eps_sample(Psample: np.ndarray, S: float, n_full: int) -> np.float32:
    """Epsilon from a sample of m points: the fraction S/(n_full-1) of pairs must lie within eps."""
    m = Psample.shape[0]
    K = int(round(S / (n_full - 1) * (m * (m - 1) // 2)))
    return eps_for_pair_rank(all_pairs_dist2(Psample), max(K, 1))


# ---------------------------------------------------------------------------------------------
# parity rule and the paper's accuracy measures
# ---------------------------------------------------------------------------------------------

def boundary_band(D2, eps, rel: float = 1e-3):
    """True where the FP64 distance lies within a relative `rel` of epsilon (either side)."""
    e = float(np.float32(eps))
    return np.abs(np.sqrt(np.asarray(D2, dtype=np.float64)) - e) <= rel * e


def pair_keys(pairs: np.ndarray) -> np.ndarray:
    p = np.asarray(pairs).astype(np.uint64)
    return (p[:, 0] << np.uint64(32)) | p[:, 1]


def overlap_accuracy(n: int, pairs_a: np.ndarray, pairs_b: np.ndarray) -> float:
    """Eq. 3: mean over points of |N_i^a intersect N_i^b| / |N_i^a union N_i^b|.

    Neighbour sets exclude the point itself; pairs are unordered (i<j) and count for both ends.
    A point with no neighbour in either set scores 1.
    """
    def nonself(p):
        p = np.asarray(p)
        return p[p[:, 0] != p[:, 1]]
    a, b = nonself(pairs_a), nonself(pairs_b)
    ka, kb = pair_keys(a), pair_keys(b)
    both = np.intersect1d(ka, kb)
    def per_point(keys):
        i = (keys >> np.uint64(32)).astype(np.int64)
        j = (keys & np.uint64(0xFFFFFFFF)).astype(np.int64)
        return np.bincount(i, minlength=n) + np.bincount(j, minlength=n)
    inter = per_point(both).astype(np.float64)
    union = per_point(ka) + per_point(kb) - inter
    score = np.ones(n, dtype=np.float64)
    nz = union > 0
    score[nz] = inter[nz] / union[nz]
    return float(score.mean())


def distance_error_stats(d2_test, d2_ref) -> tuple[float, float]:
    """Mean and standard deviation of dist_test - dist_ref over common pairs (Section 4.5)."""
    e = np.sqrt(np.maximum(np.asarray(d2_test, dtype=np.float64), 0.0)) - np.sqrt(np.asarray(d2_ref, dtype=np.float64))
    return float(e.mean()), float(e.std())
