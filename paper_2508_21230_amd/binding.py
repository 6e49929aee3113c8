"""Thin Python binding of the C ABI in include/ejoin.h.

Argument marshalling only: every step of the join runs in the HIP kernels of libejoin.so.
PyTorch supplies device memory and streams.  There is no CPU fallback: if the library is not
built or no gfx950 device is present, the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

EJOIN_OK = 0
_libs: dict = {}


class EJoinError(RuntimeError):
    pass


def load_library(path: str | None = None) -> C.CDLL:
    """dlopen libejoin.so (building it first only if it has never been built).

    `path` names another build of the same source (the ablation variants of build.build_ablations)."""
    key = os.path.abspath(path) if path else _build.LIB
    if key in _libs:
        return _libs[key]
    if path is None and not os.path.exists(_build.LIB):
        _build.build_library()
    lib = C.CDLL(key)
    vp, i64, i32, u64, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_float
    lib.ejoin_create.restype = C.c_int
    lib.ejoin_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.ejoin_destroy.restype = C.c_int
    lib.ejoin_destroy.argtypes = [vp]
    lib.ejoin_reserve.restype = C.c_int
    lib.ejoin_reserve.argtypes = [vp, i64, i32]
    lib.ejoin_strerror.restype = C.c_char_p
    lib.ejoin_strerror.argtypes = [C.c_int]
    lib.ejoin_last_hip_error.restype = C.c_char_p
    lib.ejoin_last_hip_error.argtypes = [vp]
    lib.ejoin_norms.restype = C.c_int
    lib.ejoin_norms.argtypes = [vp, vp, i64, i32, i64, vp, vp]
    lib.ejoin_selfjoin_count.restype = C.c_int
    lib.ejoin_selfjoin_count.argtypes = [vp, vp, i64, i32, i64, f32, vp, vp, vp]
    lib.ejoin_selfjoin_pairs.restype = C.c_int
    lib.ejoin_selfjoin_pairs.argtypes = [vp, vp, i64, i32, i64, f32, vp, vp, u64, vp, vp]
    lib.ejoin_selfjoin_pairs_to_host.restype = C.c_int
    lib.ejoin_selfjoin_pairs_to_host.argtypes = [vp, vp, i64, i32, i64, f32, vp, vp, u64, i32, vp, vp, C.POINTER(u64), vp]
    lib.ejoin_selfjoin_pairs_noalloc.restype = C.c_int
    lib.ejoin_selfjoin_pairs_noalloc.argtypes = [vp, vp, i64, i32, i64, f32, vp, vp, u64, vp, vp]
    lib.ejoin_selfjoin_count_f32.restype = C.c_int
    lib.ejoin_selfjoin_count_f32.argtypes = [vp, vp, i64, i32, i64, f32, vp, vp, vp]
    lib.ejoin_selfjoin_pairs_f32.restype = C.c_int
    lib.ejoin_selfjoin_pairs_f32.argtypes = [vp, vp, i64, i32, i64, f32, vp, vp, u64, vp, vp]
    lib.ejoin_set_create.restype = C.c_int
    lib.ejoin_set_create.argtypes = [vp, vp, i64, i32, i64, vp, C.POINTER(vp)]
    lib.ejoin_set_destroy.restype = C.c_int
    lib.ejoin_set_destroy.argtypes = [vp]
    lib.ejoin_set_join_pairs.restype = C.c_int
    lib.ejoin_set_join_pairs.argtypes = [vp, vp, vp, i64, i64, f32, vp, vp, u64, vp, vp]
    lib.ejoin_set_join_count.restype = C.c_int
    lib.ejoin_set_join_count.argtypes = [vp, vp, vp, i64, i64, f32, vp, vp, vp, vp]
    lib.ejoin_join_pairs.restype = C.c_int
    lib.ejoin_join_pairs.argtypes = [vp, vp, i64, i64, vp, i64, i64, i32, f32, vp, vp, u64, vp, vp]
    lib.ejoin_join_count.restype = C.c_int
    lib.ejoin_join_count.argtypes = [vp, vp, i64, i64, vp, i64, i64, i32, f32, vp, vp, vp, vp]
    lib.ejoin_tiles_evaluated2.restype = i64
    lib.ejoin_tiles_evaluated2.argtypes = [i64, i64]
    lib.ejoin_convert_f32.restype = C.c_int
    lib.ejoin_convert_f32.argtypes = [vp, vp, i64, i32, i64, vp, f32, vp, i64, vp]
    lib.ejoin_dist2_tile.restype = C.c_int
    lib.ejoin_dist2_tile.argtypes = [vp, vp, i64, i32, i64, i64, i64, i32, i32, vp, vp]
    lib.ejoin_status.restype = C.c_int
    lib.ejoin_status.argtypes = [vp, C.POINTER(C.c_int)]
    lib.ejoin_set_profiling.restype = C.c_int
    lib.ejoin_set_profiling.argtypes = [vp, C.c_int]
    lib.ejoin_last_kernel_ms.restype = C.c_int
    lib.ejoin_last_kernel_ms.argtypes = [vp, C.POINTER(f32), C.POINTER(f32)]
    lib.ejoin_tiles_evaluated.restype = i64
    lib.ejoin_tiles_evaluated.argtypes = [i64]
    _libs[key] = lib
    return lib


def tiles_evaluated(n: int) -> int:
    return int(load_library().ejoin_tiles_evaluated(int(n)))


def tiles_evaluated2(n_p: int, n_q: int) -> int:
    return int(load_library().ejoin_tiles_evaluated2(int(n_p), int(n_q)))


class EJoin:
    """One context (ejoin_ctx) on one GPU.  Methods mirror the C entry points."""

    def __init__(self, device: int = 0, lib_path: str | None = None):
        if not torch.cuda.is_available():
            raise EJoinError("no GPU visible: the epsilon self-join has no CPU path")
        self._lib = load_library(lib_path)
        self.device = torch.device("cuda", device)
        h = C.c_void_p()
        self._check(self._lib.ejoin_create(C.byref(h), device), None)
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            self._lib.ejoin_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: the modules this needs may already be gone
            pass

    def _check(self, rc: int, h):
        if rc != EJOIN_OK:
            msg = self._lib.ejoin_strerror(rc).decode()
            if h:
                extra = self._lib.ejoin_last_hip_error(h).decode()
                if extra:
                    msg += " [" + extra + "]"
            raise EJoinError(f"ejoin error {rc}: {msg}")

    @staticmethod
    def _stream():
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def _x(self, X: torch.Tensor, d):
        if X.dtype not in (torch.float16, torch.int16, torch.uint16):
            raise EJoinError("X must hold fp16 values (torch.float16, or int16/uint16 bit patterns)")
        if X.dim() != 2 or not X.is_cuda or X.stride(1) != 1:
            raise EJoinError("X must be a 2-D device tensor with contiguous rows")
        n, width = X.shape
        ld = X.stride(0) if n > 1 else max(X.stride(0), width)
        d = width if d is None else int(d)
        return n, d, ld

    def reserve(self, n: int, d: int):
        self._check(self._lib.ejoin_reserve(self._h, int(n), int(d)), self._h)

    def convert_f32(self, X32: torch.Tensor, scale: float = 1.0, center: torch.Tensor | None = None) -> torch.Tensor:
        """FP32 (n, d) device tensor -> FP16 (n, roundup(d, 64)) device tensor: fp16(scale * (x - center)), zero padded."""
        if X32.dtype != torch.float32 or X32.dim() != 2 or not X32.is_cuda or X32.stride(1) != 1:
            raise EJoinError("X32 must be a 2-D float32 device tensor with contiguous rows")
        n, d = X32.shape
        cptr = None
        if center is not None:
            if center.dtype != torch.float32 or center.numel() != d or not center.is_cuda or not center.is_contiguous():
                raise EJoinError("center must be a contiguous float32 device tensor of d elements")
            cptr = center.data_ptr()
        ld16 = (d + 63) // 64 * 64
        out = torch.empty((n, ld16), dtype=torch.float16, device=X32.device)
        self._check(self._lib.ejoin_convert_f32(self._h, X32.data_ptr(), n, d, X32.stride(0), cptr, float(scale), out.data_ptr(), ld16,
                                                self._stream()), self._h)
        return out

    def norms(self, X: torch.Tensor, d: int | None = None) -> torch.Tensor:
        n, d, ld = self._x(X, d)
        s = torch.empty(n, dtype=torch.float32, device=X.device)
        self._check(self._lib.ejoin_norms(self._h, X.data_ptr(), n, d, ld, s.data_ptr(), self._stream()), self._h)
        return s

    def selfjoin_count(self, X: torch.Tensor, eps: float, d: int | None = None, counts: torch.Tensor | None = None,
                       total: torch.Tensor | None = None):
        """Returns (counts int32[n] holding u32 values, total int64[1]) -- device tensors, stream-ordered."""
        n, d, ld = self._x(X, d)
        if counts is None:
            counts = torch.empty(n, dtype=torch.int32, device=X.device)
        if total is None:
            total = torch.empty(1, dtype=torch.int64, device=X.device)
        self._check(self._lib.ejoin_selfjoin_count(self._h, X.data_ptr(), n, d, ld, float(eps), counts.data_ptr(),
                                                   total.data_ptr(), self._stream()), self._h)
        return counts, total

    def selfjoin_pairs(self, X: torch.Tensor, eps: float, capacity: int, d: int | None = None, with_dist2: bool = True,
                       pairs: torch.Tensor | None = None, dist2: torch.Tensor | None = None,
                       n_pairs: torch.Tensor | None = None):
        """Returns (pairs int32[capacity, 2] holding u32 values, dist2 float32[capacity] or None, n_pairs int64[1])."""
        n, d, ld = self._x(X, d)
        capacity = int(capacity)
        if pairs is None:
            pairs = torch.empty((max(capacity, 1), 2), dtype=torch.int32, device=X.device)
        if dist2 is None and with_dist2:
            dist2 = torch.empty(max(capacity, 1), dtype=torch.float32, device=X.device)
        if n_pairs is None:
            n_pairs = torch.empty(1, dtype=torch.int64, device=X.device)
        self._check(self._lib.ejoin_selfjoin_pairs(self._h, X.data_ptr(), n, d, ld, float(eps), pairs.data_ptr(),
                                                   dist2.data_ptr() if dist2 is not None else None, capacity,
                                                   n_pairs.data_ptr(), self._stream()), self._h)
        return pairs, dist2, n_pairs

    def selfjoin_pairs_to_host(self, X: torch.Tensor, eps: float, batches: int, pairs: torch.Tensor, dist2: torch.Tensor | None,
                               host_pairs: torch.Tensor, host_dist2: torch.Tensor | None, d: int | None = None) -> int:
        """ejoin_selfjoin_pairs_to_host: the join in `batches` launches, each batch's pairs copied to the host tensors
        (CPU, ideally pinned: int32[capacity, 2], float32[capacity] or None) while the next one computes.  Blocks;
        returns the number of pairs found."""
        n, d, ld = self._x(X, d)
        capacity = int(pairs.shape[0])
        if host_pairs.is_cuda or host_pairs.shape[0] < capacity or not host_pairs.is_contiguous():
            raise EJoinError("host_pairs must be a contiguous CPU tensor of at least `capacity` pairs")
        if (dist2 is None) != (host_dist2 is None):
            raise EJoinError("dist2 and host_dist2 go together")
        found = C.c_uint64()
        self._check(self._lib.ejoin_selfjoin_pairs_to_host(self._h, X.data_ptr(), n, d, ld, float(eps), pairs.data_ptr(),
                                                           dist2.data_ptr() if dist2 is not None else None, capacity, int(batches),
                                                           host_pairs.data_ptr(), host_dist2.data_ptr() if host_dist2 is not None else None,
                                                           C.byref(found), self._stream()), self._h)
        return int(found.value)

    def selfjoin_pairs_noalloc(self, X: torch.Tensor, eps: float, pairs: torch.Tensor, dist2: torch.Tensor | None,
                               n_pairs: torch.Tensor, d: int | None = None):
        """ejoin_selfjoin_pairs_noalloc: the caller supplies every output (pairs int32[capacity, 2], dist2 float32[capacity]
        or None, n_pairs int64[1]); neither the library nor this method allocates device memory."""
        n, d, ld = self._x(X, d)
        capacity = int(pairs.shape[0])
        if dist2 is not None and dist2.shape[0] < capacity:
            raise EJoinError("dist2 must hold as many entries as pairs")
        self._check(self._lib.ejoin_selfjoin_pairs_noalloc(self._h, X.data_ptr(), n, d, ld, float(eps), pairs.data_ptr(),
                                                           dist2.data_ptr() if dist2 is not None else None, capacity,
                                                           n_pairs.data_ptr(), self._stream()), self._h)
        return pairs, dist2, n_pairs

    @staticmethod
    def _x32(X32: torch.Tensor):
        if X32.dtype != torch.float32 or X32.dim() != 2 or not X32.is_cuda or X32.stride(1) != 1:
            raise EJoinError("X32 must be a 2-D float32 device tensor with contiguous rows")
        return X32.shape[0], X32.shape[1], X32.stride(0)

    def selfjoin_pairs_f32(self, X32: torch.Tensor, eps: float, capacity: int, with_dist2: bool = True,
                           pairs: torch.Tensor | None = None, dist2: torch.Tensor | None = None, n_pairs: torch.Tensor | None = None):
        """Split-FP16 self-join of FP32 rows; returns like selfjoin_pairs."""
        n, d, ld = self._x32(X32)
        capacity = int(capacity)
        if pairs is None:
            pairs = torch.empty((max(capacity, 1), 2), dtype=torch.int32, device=X32.device)
        if dist2 is None and with_dist2:
            dist2 = torch.empty(max(capacity, 1), dtype=torch.float32, device=X32.device)
        if n_pairs is None:
            n_pairs = torch.empty(1, dtype=torch.int64, device=X32.device)
        self._check(self._lib.ejoin_selfjoin_pairs_f32(self._h, X32.data_ptr(), n, d, ld, float(eps), pairs.data_ptr(),
                                                       dist2.data_ptr() if dist2 is not None else None, capacity,
                                                       n_pairs.data_ptr(), self._stream()), self._h)
        return pairs, dist2, n_pairs

    def selfjoin_count_f32(self, X32: torch.Tensor, eps: float, counts: torch.Tensor | None = None, total: torch.Tensor | None = None):
        """Split-FP16 neighbour counts of FP32 rows; returns like selfjoin_count."""
        n, d, ld = self._x32(X32)
        if counts is None:
            counts = torch.empty(n, dtype=torch.int32, device=X32.device)
        if total is None:
            total = torch.empty(1, dtype=torch.int64, device=X32.device)
        self._check(self._lib.ejoin_selfjoin_count_f32(self._h, X32.data_ptr(), n, d, ld, float(eps), counts.data_ptr(),
                                                       total.data_ptr(), self._stream()), self._h)
        return counts, total

    def prepare(self, X: torch.Tensor, d: int | None = None) -> "EJoinSet":
        """Prepared point set (ejoin_set_create): pack X and compute its norms once, join query batches against it."""
        return EJoinSet(self, X, d)

    def join_pairs(self, P: torch.Tensor, Q: torch.Tensor, eps: float, capacity: int, d: int | None = None, with_dist2: bool = True,
                   pairs: torch.Tensor | None = None, dist2: torch.Tensor | None = None, n_pairs: torch.Tensor | None = None):
        """Two-set join; returns (pairs int32[capacity, 2]: (index into P, index into Q), dist2 or None, n_pairs int64[1])."""
        n_p, d_p, ldp = self._x(P, d)
        n_q, d_q, ldq = self._x(Q, d)
        if d_p != d_q:
            raise EJoinError("P and Q must have the same number of coordinates")
        capacity = int(capacity)
        if pairs is None:
            pairs = torch.empty((max(capacity, 1), 2), dtype=torch.int32, device=P.device)
        if dist2 is None and with_dist2:
            dist2 = torch.empty(max(capacity, 1), dtype=torch.float32, device=P.device)
        if n_pairs is None:
            n_pairs = torch.empty(1, dtype=torch.int64, device=P.device)
        self._check(self._lib.ejoin_join_pairs(self._h, P.data_ptr(), n_p, ldp, Q.data_ptr(), n_q, ldq, d_p, float(eps), pairs.data_ptr(),
                                               dist2.data_ptr() if dist2 is not None else None, capacity, n_pairs.data_ptr(),
                                               self._stream()), self._h)
        return pairs, dist2, n_pairs

    def join_count(self, P: torch.Tensor, Q: torch.Tensor, eps: float, d: int | None = None, want_counts_q: bool = True):
        """Two-set join counts; returns (counts_p int32[np], counts_q int32[nq] or None, total int64[1])."""
        n_p, d_p, ldp = self._x(P, d)
        n_q, d_q, ldq = self._x(Q, d)
        if d_p != d_q:
            raise EJoinError("P and Q must have the same number of coordinates")
        cp = torch.empty(n_p, dtype=torch.int32, device=P.device)
        cq = torch.empty(n_q, dtype=torch.int32, device=P.device) if want_counts_q else None
        total = torch.empty(1, dtype=torch.int64, device=P.device)
        self._check(self._lib.ejoin_join_count(self._h, P.data_ptr(), n_p, ldp, Q.data_ptr(), n_q, ldq, d_p, float(eps), cp.data_ptr(),
                                               cq.data_ptr() if cq is not None else None, total.data_ptr(), self._stream()), self._h)
        return cp, cq, total

    def dist2_tile(self, X: torch.Tensor, i0: int, j0: int, rows: int, cols: int, d: int | None = None) -> torch.Tensor:
        n, d, ld = self._x(X, d)
        out = torch.empty((rows, cols), dtype=torch.float32, device=X.device)
        self._check(self._lib.ejoin_dist2_tile(self._h, X.data_ptr(), n, d, ld, int(i0), int(j0), int(rows), int(cols),
                                               out.data_ptr(), self._stream()), self._h)
        return out

    def status(self) -> int:
        """Device status of the last join / dense-tile call (0 = ok); synchronises."""
        st = C.c_int()
        self._check(self._lib.ejoin_status(self._h, C.byref(st)), self._h)
        return int(st.value)

    def set_profiling(self, on: bool):
        self._check(self._lib.ejoin_set_profiling(self._h, 1 if on else 0), self._h)

    def last_kernel_ms(self) -> tuple[float, float]:
        a, b = C.c_float(), C.c_float()
        self._check(self._lib.ejoin_last_kernel_ms(self._h, C.byref(a), C.byref(b)), self._h)
        return float(a.value), float(b.value)


class EJoinSet:
    """A prepared point set (ejoin_set).  Joins that use the same set must not overlap."""

    def __init__(self, ej: EJoin, X: torch.Tensor, d: int | None = None):
        self._ej = ej
        self.n, self.d, ld = ej._x(X, d)
        h = C.c_void_p()
        ej._check(ej._lib.ejoin_set_create(ej._h, X.data_ptr(), self.n, self.d, ld, ej._stream(), C.byref(h)), ej._h)
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and getattr(self._ej, "_h", None):
            torch.cuda.synchronize(self._ej.device)
            self._ej._lib.ejoin_set_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def join_pairs(self, Q: torch.Tensor, eps: float, capacity: int, with_dist2: bool = True, pairs: torch.Tensor | None = None,
                   dist2: torch.Tensor | None = None, n_pairs: torch.Tensor | None = None):
        """Like EJoin.join_pairs with P = this set."""
        ej = self._ej
        n_q, d_q, ldq = ej._x(Q, self.d)
        capacity = int(capacity)
        if pairs is None:
            pairs = torch.empty((max(capacity, 1), 2), dtype=torch.int32, device=Q.device)
        if dist2 is None and with_dist2:
            dist2 = torch.empty(max(capacity, 1), dtype=torch.float32, device=Q.device)
        if n_pairs is None:
            n_pairs = torch.empty(1, dtype=torch.int64, device=Q.device)
        ej._check(ej._lib.ejoin_set_join_pairs(ej._h, self._h, Q.data_ptr(), n_q, ldq, float(eps), pairs.data_ptr(),
                                               dist2.data_ptr() if dist2 is not None else None, capacity, n_pairs.data_ptr(),
                                               ej._stream()), ej._h)
        return pairs, dist2, n_pairs

    def join_count(self, Q: torch.Tensor, eps: float, want_counts_q: bool = True):
        """Like EJoin.join_count with P = this set: (counts_p, counts_q or None, total)."""
        ej = self._ej
        n_q, d_q, ldq = ej._x(Q, self.d)
        counts_p = torch.empty(self.n, dtype=torch.int32, device=Q.device)
        counts_q = torch.empty(n_q, dtype=torch.int32, device=Q.device) if want_counts_q else None
        total = torch.empty(1, dtype=torch.int64, device=Q.device)
        ej._check(ej._lib.ejoin_set_join_count(ej._h, self._h, Q.data_ptr(), n_q, ldq, float(eps), counts_p.data_ptr(),
                                               counts_q.data_ptr() if counts_q is not None else None, total.data_ptr(),
                                               ej._stream()), ej._h)
        return counts_p, counts_q, total
