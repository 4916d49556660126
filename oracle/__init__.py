"""CPU oracle for the mixed-precision weight format (test infrastructure, not product code).

Thin ctypes marshalling around oracle/mpq_oracle.c; all arithmetic lives in the C file.
Only tests/, the smoke check and the benchmark's cpu_baseline leg import this package.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


class OrcDesc(C.Structure):
    _fields_ = [("N", C.c_int32), ("K", C.c_int32), ("g1", C.c_int32), ("g2", C.c_int32),
                ("g2_axis", C.c_int32)]


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_half_to_float.restype = C.c_float
        L.orc_half_to_float.argtypes = [C.c_uint16]
        L.orc_float_to_half.restype = C.c_uint16
        L.orc_float_to_half.argtypes = [C.c_float]
        L.orc_scale_dequant.restype = C.c_uint16
        L.orc_scale_dequant.argtypes = [C.c_uint8, C.c_uint16, C.c_uint16]
        L.orc_weight_dequant.restype = C.c_uint16
        L.orc_weight_dequant.argtypes = [C.c_uint8, C.c_uint8, C.c_uint16]
        L.orc_add_outlier.restype = C.c_uint16
        L.orc_add_outlier.argtypes = [C.c_uint16, C.c_uint16]
        L.orc_validate.restype = C.c_int
        L.orc_validate.argtypes = [C.POINTER(OrcDesc)] + [C.c_void_p] * 4
        L.orc_scales.restype = None
        L.orc_scales.argtypes = [C.POINTER(OrcDesc)] + [C.c_void_p] * 4
        L.orc_dequant.restype = None
        L.orc_dequant.argtypes = [C.POINTER(OrcDesc)] + [C.c_void_p] * 8 + [C.c_int, C.c_void_p]
        L.orc_gemm_rows.restype = None
        L.orc_gemm_rows.argtypes = ([C.POINTER(OrcDesc)] + [C.c_void_p] * 9 +
                                    [C.c_int32, C.c_int64, C.c_int64, C.c_int, C.c_void_p])
        for name in ("orc_avg_bits_first_order", "orc_avg_bits_second_order", "orc_avg_bits_mixed",
                     "orc_outlier_bits", "orc_avg_bits_stored"):
            getattr(L, name).restype = C.c_double
        L.orc_avg_bits_first_order.argtypes = [C.c_int, C.c_int]
        L.orc_avg_bits_second_order.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_avg_bits_mixed.argtypes = [C.c_double, C.c_int, C.c_int, C.c_int]
        L.orc_outlier_bits.argtypes = [C.c_double]
        L.orc_avg_bits_stored.argtypes = [C.POINTER(OrcDesc), C.c_int32, C.c_int64]
        L.orc_clip_scales.restype = None
        L.orc_clip_scales.argtypes = [C.POINTER(OrcDesc)] + [C.c_void_p] * 3
        L.orc_validate_aligned.restype = C.c_int
        L.orc_validate_aligned.argtypes = [C.POINTER(OrcDesc)] + [C.c_void_p] * 4
        L.orc_avg_bits_stored_aligned.restype = C.c_double
        L.orc_avg_bits_stored_aligned.argtypes = [C.POINTER(OrcDesc), C.c_int32, C.c_int64]
        L.orc_max_threads.restype = C.c_int
        _LIB = L
    return _LIB


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return np.array(a, dtype=dtype, order="C", copy=True)


def _desc(N, K, g1, g2, g2_axis=0):
    return OrcDesc(int(N), int(K), int(g1), int(g2), int(g2_axis))


class Matrix:
    """Holds contiguous copies of the logical arrays of one matrix for the C calls."""

    def __init__(self, N, K, g1, g2, is4, codes, s_int, z1, s2, z2, row_ptr, col, val, g2_axis=0):
        self.d = _desc(N, K, g1, g2, g2_axis)
        self.N, self.K, self.g1, self.g2, self.g2_axis = int(N), int(K), int(g1), int(g2), int(g2_axis)
        self.G = self.K // self.g1
        self.is4 = _c(is4, np.uint8)
        self.codes = _c(codes, np.uint8).reshape(self.N, self.K)
        self.s_int = _c(s_int, np.uint8).reshape(self.N, self.G)
        self.z1 = _c(z1, np.uint8).reshape(self.N, self.G)
        self.s2 = _c(s2, np.uint16)
        self.z2 = _c(z2, np.uint16)
        self.row_ptr = _c(row_ptr, np.int32)
        self.col = _c(col, np.uint16)
        self.val = _c(val, np.uint16)

    @classmethod
    def from_logical(cls, lg, g2_axis=None):
        if g2_axis is None:
            g2_axis = getattr(lg.spec, "g2_axis", 0)
        s = lg.spec
        return cls(s.N, s.K, s.g1, s.g2, lg.is4, lg.codes, lg.s_int, lg.z1, lg.s2, lg.z2,
                   lg.row_ptr, lg.col, lg.val, g2_axis)

    def validate(self) -> int:
        return lib().orc_validate(C.byref(self.d), _p(self.is4), _p(self.codes), _p(self.row_ptr), _p(self.col))

    def scales(self) -> np.ndarray:
        out = np.empty((self.N, self.G), dtype=np.uint16)
        lib().orc_scales(C.byref(self.d), _p(self.s_int), _p(self.s2), _p(self.z2), _p(out))
        return out

    def dequant(self, add_outliers: bool = False) -> np.ndarray:
        """Row-major N x K fp16 bit patterns."""
        out = np.empty((self.N, self.K), dtype=np.uint16)
        lib().orc_dequant(C.byref(self.d), _p(self.codes), _p(self.s_int), _p(self.z1), _p(self.s2),
                          _p(self.z2), _p(self.row_ptr), _p(self.col), _p(self.val),
                          int(bool(add_outliers)), _p(out))
        return out

    def gemm(self, X_bits, rows=None, threads: int = 1) -> np.ndarray:
        """Y[M, N] in binary64 (only rows [rows[0], rows[1]) are filled when `rows` is given)."""
        X = _c(X_bits, np.uint16)
        if X.ndim == 1:
            X = X.reshape(1, -1)
        M = X.shape[0]
        assert X.shape[1] == self.K
        Y = np.zeros((M, self.N), dtype=np.float64)
        lo, hi = (0, self.N) if rows is None else rows
        lib().orc_gemm_rows(C.byref(self.d), _p(self.codes), _p(self.s_int), _p(self.z1), _p(self.s2),
                            _p(self.z2), _p(self.row_ptr), _p(self.col), _p(self.val), _p(X),
                            M, int(lo), int(hi), int(threads), _p(Y))
        return Y


def half_to_float(h: int) -> float:
    return float(lib().orc_half_to_float(int(h)))


def float_to_half(f: float) -> int:
    return int(lib().orc_float_to_half(C.c_float(f)))


def scale_dequant(s_int: int, z2: int, s2: int) -> int:
    return int(lib().orc_scale_dequant(int(s_int), int(z2), int(s2)))


def weight_dequant(code: int, z1: int, s1: int) -> int:
    return int(lib().orc_weight_dequant(int(code), int(z1), int(s1)))


def add_outlier(w: int, val: int) -> int:
    return int(lib().orc_add_outlier(int(w), int(val)))


def avg_bits_first_order(nbits, g1):
    return float(lib().orc_avg_bits_first_order(nbits, g1))


def avg_bits_second_order(nbits, ns, g1, g2):
    return float(lib().orc_avg_bits_second_order(nbits, ns, g1, g2))


def avg_bits_mixed(alpha, ns, g1, g2):
    return float(lib().orc_avg_bits_mixed(alpha, ns, g1, g2))


def outlier_bits(ratio):
    return float(lib().orc_outlier_bits(ratio))


def avg_bits_stored(N, K, g1, g2, n4, nnz, g2_axis=0):
    d = _desc(N, K, g1, g2, g2_axis)
    return float(lib().orc_avg_bits_stored(C.byref(d), int(n4), int(nnz)))


def clip_scales(N, K, g1, is4, s_int) -> np.ndarray:
    """Scale codes clipped to the fields of the aligned metadata format (Sec. 3.3 "Scale Clipping")."""
    d = _desc(N, K, g1, 1)
    is4 = _c(is4, np.uint8)
    s_in = _c(s_int, np.uint8)
    out = np.zeros_like(s_in)
    lib().orc_clip_scales(C.byref(d), _p(is4), _p(s_in), _p(out))
    return out


def validate_aligned(N, K, g1, g2, is4, s_int, z1, z2, g2_axis=0) -> int:
    d = _desc(N, K, g1, g2, g2_axis)
    return int(lib().orc_validate_aligned(C.byref(d), _p(_c(is4, np.uint8)), _p(_c(s_int, np.uint8)), _p(_c(z1, np.uint8)),
                                          _p(_c(z2, np.uint16))))


def avg_bits_stored_aligned(N, K, g1, g2, n4, nnz, g2_axis=0):
    d = _desc(N, K, g1, g2, g2_axis)
    return float(lib().orc_avg_bits_stored_aligned(C.byref(d), int(n4), int(nnz)))


def max_threads() -> int:
    return int(lib().orc_max_threads())
