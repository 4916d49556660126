"""Python binding of libmpq (2/4/16-bit mixed-precision weights on MI355X).

Argument marshalling only: every function here forwards to the C entry point of the same name
declared in include/mpq.h.  There is no Python or CPU fallback; if the compiled library is
missing the import of a device function raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmpq.so")
HEADER_BYTES = 256
MAX_M = 32

STATUS_NAMES = ["MPQ_OK", "MPQ_ERR_NULL", "MPQ_ERR_SHAPE", "MPQ_ERR_ALIGN", "MPQ_ERR_CODE_RANGE",
                "MPQ_ERR_OUTLIER_IN_4BIT", "MPQ_ERR_CSR", "MPQ_ERR_BLOB", "MPQ_ERR_SIZE",
                "MPQ_ERR_UNSUPPORTED", "MPQ_ERR_HIP"]
(MPQ_OK, MPQ_ERR_NULL, MPQ_ERR_SHAPE, MPQ_ERR_ALIGN, MPQ_ERR_CODE_RANGE, MPQ_ERR_OUTLIER_IN_4BIT,
 MPQ_ERR_CSR, MPQ_ERR_BLOB, MPQ_ERR_SIZE, MPQ_ERR_UNSUPPORTED, MPQ_ERR_HIP) = range(11)

EXPORTS = ["mpq_status_str", "mpq_avg_bits", "mpq_quantize_host", "mpq_quantize_outlier_capacity", "mpq_packed_size",
           "mpq_pack_host", "mpq_blob_info", "mpq_blob_tiles", "mpq_dequant", "mpq_gemv", "mpq_gemv_multi", "mpq_gemm_workspace_size",
           "mpq_gemm", "mpq_gemm_planned", "mpq_gemm_workspace_size_planned", "mpq_gemm_static", "mpq_stream_probe"]
STATIC_SCRATCH_BYTES = 32 << 20
(KERNEL_GEMV_PLANES, KERNEL_GEMV_DECODE, KERNEL_BATCH_RESIDENT, KERNEL_BATCH_RANGES) = (1, 2, 3, 4)
MAX_MULTI = 8


class MpqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name} ({status_str(status)})")


class Desc(C.Structure):
    _fields_ = [("N", C.c_int32), ("K", C.c_int32), ("g1", C.c_int32), ("g2", C.c_int32),
                ("g2_axis", C.c_int32), ("meta", C.c_int32)]


class Plan(C.Structure):
    """mpq_plan: 0 in a field = the library's own choice."""
    _fields_ = [(n, C.c_int32) for n in ("gemv_path", "gemv_waves", "gemv_tiles", "batch_waves", "max_workgroups",
                                         "large_batch", "lb_min_ranges", "lb_tiles", "lb_older16", "gemv_older")] + \
               [("reserved", C.c_int32 * 6)]


class Report(C.Structure):
    """mpq_report: what a planned call enqueued."""
    _fields_ = [(n, C.c_int32) for n in ("kernel", "launches", "waves", "tiles_per_workgroup", "workgroups")] + \
               [("reserved", C.c_int32 * 3)]


class LogicalOutPtrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("is4", "codes", "s_int", "z1", "s2", "z2", "row_ptr", "col", "val")]


class LogicalPtrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("is4", "codes", "s_int", "z1", "s2", "z2", "row_ptr", "col", "val")]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # PyTorch ships its own copy of the HIP runtime.  The caller's device memory and streams come
        # from that copy, so it has to be the one this library binds to: load torch first (a library
        # loaded before torch would pull in the system's runtime, and launches on torch's streams
        # through a second runtime fail).
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        L.mpq_status_str.restype = C.c_char_p
        L.mpq_status_str.argtypes = [C.c_int]
        L.mpq_avg_bits.restype = C.c_double
        L.mpq_avg_bits.argtypes = [C.POINTER(Desc), C.c_int32, C.c_int64, C.c_int, C.c_int]
        L.mpq_quantize_host.restype = C.c_int
        L.mpq_quantize_host.argtypes = [C.POINTER(Desc), C.c_void_p, C.c_int32, C.c_double,
                                        C.POINTER(LogicalOutPtrs), C.c_int64, C.POINTER(C.c_int64)]
        L.mpq_packed_size.restype = C.c_int
        L.mpq_packed_size.argtypes = [C.POINTER(Desc), C.c_void_p, C.c_void_p, C.POINTER(C.c_size_t)]
        L.mpq_pack_host.restype = C.c_int
        L.mpq_pack_host.argtypes = [C.POINTER(Desc), C.POINTER(LogicalPtrs), C.c_void_p, C.c_size_t]
        L.mpq_blob_info.restype = C.c_int
        L.mpq_blob_info.argtypes = [C.c_void_p, C.POINTER(Desc), C.POINTER(C.c_int64),
                                    C.POINTER(C.c_int32), C.POINTER(C.c_uint64)]
        L.mpq_blob_tiles.restype = C.c_int
        L.mpq_blob_tiles.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_int32)]
        L.mpq_dequant.restype = C.c_int
        L.mpq_dequant.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.mpq_gemv.restype = C.c_int
        L.mpq_gemv.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.mpq_gemv_multi.restype = C.c_int
        L.mpq_gemv_multi.argtypes = [C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                     C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p]
        L.mpq_gemm.restype = C.c_int
        L.mpq_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t,
                               C.c_void_p]
        L.mpq_gemm_workspace_size.restype = C.c_int
        L.mpq_gemm_workspace_size.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]
        L.mpq_gemm_planned.restype = C.c_int
        L.mpq_gemm_planned.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t,
                                       C.c_void_p, C.POINTER(Plan), C.POINTER(Report)]
        L.mpq_gemm_workspace_size_planned.restype = C.c_int
        L.mpq_gemm_workspace_size_planned.argtypes = [C.c_void_p, C.c_int32, C.POINTER(Plan), C.POINTER(C.c_size_t)]
        L.mpq_gemm_static.restype = C.c_int
        L.mpq_gemm_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.mpq_stream_probe.restype = C.c_int
        L.mpq_stream_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.mpq_quantize_outlier_capacity.restype = C.c_int
        L.mpq_quantize_outlier_capacity.argtypes = [C.POINTER(Desc), C.c_int32, C.c_double, C.POINTER(C.c_int64)]
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().mpq_status_str(int(status)).decode()


def _check(status: int, where: str):
    if status != MPQ_OK:
        raise MpqError(status, where)


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


META_BYTES, META_PAPER = 0, 1


def avg_bits(N, K, g1, g2, n4, nnz, mode=0, ns_bits=4, g2_axis=0, meta=0) -> float:
    d = Desc(N, K, g1, g2, g2_axis, meta)
    return float(lib().mpq_avg_bits(C.byref(d), int(n4), int(nnz), int(mode), int(ns_bits)))


def packed_size(N, K, g1, g2, is4, row_ptr, g2_axis=0, meta=0) -> int:
    d = Desc(N, K, g1, g2, g2_axis, meta)
    is4 = _np(is4, np.uint8)
    rp = _np(row_ptr, np.int32)
    if rp.size != N + 1:
        raise MpqError(MPQ_ERR_SHAPE, "mpq_packed_size")
    out = C.c_size_t(0)
    _check(lib().mpq_packed_size(C.byref(d), is4.ctypes.data_as(C.c_void_p), rp.ctypes.data_as(C.c_void_p),
                                 C.byref(out)), "mpq_packed_size")
    return int(out.value)


def quantize(W, g1, g2, n4, p_o, g2_axis=0) -> dict:
    """mpq_quantize_host: float weights [N, K] -> dict of the logical arrays (the keyword arguments of pack)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    if W.ndim != 2:
        raise MpqError(MPQ_ERR_SHAPE, "mpq_quantize_host")
    N, K = W.shape
    d = Desc(int(N), int(K), int(g1), int(g2), int(g2_axis))
    if g1 <= 0 or g2 <= 0 or K % g1 != 0 or not 0 <= n4 <= K // g1 or not 0.0 <= p_o <= 1.0:
        raise MpqError(MPQ_ERR_SHAPE, "mpq_quantize_host")
    G = K // g1
    cap_c = C.c_int64(0)
    _check(lib().mpq_quantize_outlier_capacity(C.byref(d), int(n4), float(p_o), C.byref(cap_c)),
           "mpq_quantize_outlier_capacity")
    cap = int(cap_c.value)
    shape2 = (N, -(-G // g2)) if g2_axis == 0 else (-(-N // g2), G)
    out = dict(is4=np.zeros(G, np.uint8), codes=np.zeros((N, K), np.uint8), s_int=np.zeros((N, G), np.uint8),
               z1=np.zeros((N, G), np.uint8), s2=np.zeros(shape2, np.uint16), z2=np.zeros(shape2, np.uint16),
               row_ptr=np.zeros(N + 1, np.int32), col=np.zeros(max(cap, 1), np.uint16), val=np.zeros(max(cap, 1), np.uint16))
    ptrs = LogicalOutPtrs(**{k: v.ctypes.data for k, v in out.items()})
    nnz = C.c_int64(0)
    _check(lib().mpq_quantize_host(C.byref(d), W.ctypes.data_as(C.c_void_p), int(n4), float(p_o), C.byref(ptrs),
                                   cap, C.byref(nnz)), "mpq_quantize_host")
    out["col"], out["val"] = out["col"][: nnz.value], out["val"][: nnz.value]
    return out


@dataclass
class Packed:
    """A packed matrix on the host: `blob` (uint8 array, starts with the 256-byte header)."""
    blob: np.ndarray
    N: int
    K: int
    g1: int
    g2: int
    n4: int
    nnz: int

    @property
    def header(self) -> np.ndarray:
        return self.blob[:HEADER_BYTES]


def pack(N, K, g1, g2, is4, codes, s_int, z1, s2, z2, row_ptr, col, val, g2_axis=0, meta=0) -> Packed:
    """mpq_packed_size + mpq_pack_host on host arrays in the logical format."""
    d = Desc(int(N), int(K), int(g1), int(g2), int(g2_axis), int(meta))
    is4 = _np(is4, np.uint8)
    arrs = dict(is4=is4, codes=_np(codes, np.uint8), s_int=_np(s_int, np.uint8), z1=_np(z1, np.uint8),
                s2=_np(s2, np.uint16), z2=_np(z2, np.uint16), row_ptr=_np(row_ptr, np.int32),
                col=_np(col, np.uint16), val=_np(val, np.uint16))
    if arrs["row_ptr"].size != int(N) + 1:
        raise MpqError(MPQ_ERR_SHAPE, "mpq_pack_host")
    size = C.c_size_t(0)
    _check(lib().mpq_packed_size(C.byref(d), is4.ctypes.data_as(C.c_void_p),
                                 arrs["row_ptr"].ctypes.data_as(C.c_void_p), C.byref(size)), "mpq_packed_size")
    blob = np.empty(size.value, dtype=np.uint8)
    ptrs = LogicalPtrs(**{k: (v.ctypes.data if v.size else None) for k, v in arrs.items()})
    _check(lib().mpq_pack_host(C.byref(d), C.byref(ptrs), blob.ctypes.data_as(C.c_void_p), size.value),
           "mpq_pack_host")
    info = blob_info(blob)
    return Packed(blob, int(N), int(K), int(g1), int(g2), info["n4"], info["nnz"])


def pack_logical(lg, g2_axis=None) -> Packed:
    s = lg.spec
    if g2_axis is None:
        g2_axis = getattr(s, "g2_axis", 0)
    return pack(s.N, s.K, s.g1, s.g2, lg.is4, lg.codes, lg.s_int, lg.z1, lg.s2, lg.z2,
                lg.row_ptr, lg.col, lg.val, g2_axis, getattr(s, "meta", 0))


def blob_info(header) -> dict:
    h = _np(header, np.uint8)
    if h.size < HEADER_BYTES:
        raise MpqError(MPQ_ERR_SIZE, "mpq_blob_info")
    d = Desc()
    nnz, n4, tot = C.c_int64(0), C.c_int32(0), C.c_uint64(0)
    _check(lib().mpq_blob_info(h.ctypes.data_as(C.c_void_p), C.byref(d), C.byref(nnz), C.byref(n4),
                               C.byref(tot)), "mpq_blob_info")
    return dict(N=d.N, K=d.K, g1=d.g1, g2=d.g2, g2_axis=d.g2_axis, meta=d.meta, nnz=int(nnz.value), n4=int(n4.value),
                total_bytes=int(tot.value))


def blob_tiles(header) -> tuple:
    """mpq_blob_tiles: (offset of the first 16-row record, bytes per record, number of records)."""
    h = _np(header, np.uint8)
    off, rec, cnt = C.c_uint64(0), C.c_uint64(0), C.c_int32(0)
    _check(lib().mpq_blob_tiles(h.ctypes.data_as(C.c_void_p), C.byref(off), C.byref(rec), C.byref(cnt)), "mpq_blob_tiles")
    return int(off.value), int(rec.value), int(cnt.value)


# ----------------------------------------------------------------------------- device entry points

def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if hasattr(stream, "cuda_stream"):
        return int(stream.cuda_stream) or None
    return int(stream) or None


def _hdr_ptr(header: np.ndarray):
    h = _np(header, np.uint8)
    return h, h.ctypes.data_as(C.c_void_p)


def dequant(header, blob_dev, W_out_dev, add_outliers=False, stream=None):
    """mpq_dequant: blob_dev / W_out_dev are torch CUDA tensors (uint8 / 16-bit)."""
    h, hp = _hdr_ptr(header)
    _check(lib().mpq_dequant(hp, blob_dev.data_ptr(), W_out_dev.data_ptr(), int(bool(add_outliers)),
                             _stream_ptr(stream)), "mpq_dequant")


def gemv(header, blob_dev, x_dev, y_dev, stream=None):
    h, hp = _hdr_ptr(header)
    _check(lib().mpq_gemv(hp, blob_dev.data_ptr(), x_dev.data_ptr(), y_dev.data_ptr(),
                          _stream_ptr(stream)), "mpq_gemv")


def gemv_multi(headers, blobs_dev, xs_dev, ys_dev, stream=None):
    """mpq_gemv_multi: lists of headers (host arrays) and of CUDA tensors, one entry per product."""
    n = len(headers)
    if not (n == len(blobs_dev) == len(xs_dev) == len(ys_dev)):
        raise MpqError(MPQ_ERR_SHAPE, "mpq_gemv_multi")
    keep = [_np(h, np.uint8) for h in headers]
    arr = lambda vals: (C.c_void_p * n)(*vals)
    _check(lib().mpq_gemv_multi(n, arr([k.ctypes.data for k in keep]), arr([b.data_ptr() for b in blobs_dev]),
                                arr([x.data_ptr() for x in xs_dev]), arr([y.data_ptr() for y in ys_dev]),
                                _stream_ptr(stream)), "mpq_gemv_multi")


def gemm_workspace_size(header, M) -> int:
    """Bytes of device workspace with which gemm() runs its fastest path (0: none needed)."""
    h, hp = _hdr_ptr(header)
    n = C.c_size_t(0)
    _check(lib().mpq_gemm_workspace_size(hp, int(M), C.byref(n)), "mpq_gemm_workspace_size")
    return int(n.value)


def gemm_planned(header, blob_dev, X_dev, Y_dev, M, plan=None, stream=None, workspace=None) -> Report:
    """mpq_gemm_planned: `plan` is a Plan (or None); returns the Report of what was enqueued."""
    h, hp = _hdr_ptr(header)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rep = Report()
    _check(lib().mpq_gemm_planned(hp, blob_dev.data_ptr(), X_dev.data_ptr(), Y_dev.data_ptr(), int(M), ws_ptr, ws_bytes,
                                  _stream_ptr(stream), C.byref(plan) if plan is not None else None, C.byref(rep)),
           "mpq_gemm_planned")
    return rep


def gemm_workspace_size_planned(header, M, plan=None) -> int:
    h, hp = _hdr_ptr(header)
    n = C.c_size_t(0)
    _check(lib().mpq_gemm_workspace_size_planned(hp, int(M), C.byref(plan) if plan is not None else None, C.byref(n)),
           "mpq_gemm_workspace_size_planned")
    return int(n.value)


def gemm(header, blob_dev, X_dev, Y_dev, M, stream=None, workspace=None):
    """workspace: a device tensor (256-byte aligned) of at least gemm_workspace_size() bytes, or None."""
    h, hp = _hdr_ptr(header)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().mpq_gemm(hp, blob_dev.data_ptr(), X_dev.data_ptr(), Y_dev.data_ptr(), int(M), ws_ptr, ws_bytes,
                          _stream_ptr(stream)), "mpq_gemm")


def gemm_static(header, blob_dev, X_dev, Y_dev, M, stream=None):
    """mpq_gemm_static: the product with the library's own device scratch as workspace (no allocation)."""
    h, hp = _hdr_ptr(header)
    _check(lib().mpq_gemm_static(hp, blob_dev.data_ptr(), X_dev.data_ptr(), Y_dev.data_ptr(), int(M),
                                 _stream_ptr(stream)), "mpq_gemm_static")


def stream_probe(src_dev, nbytes=None, stream=None):
    """mpq_stream_probe: one read-only pass over a device tensor (or its first nbytes bytes)."""
    n = src_dev.numel() * src_dev.element_size() if nbytes is None else int(nbytes)
    _check(lib().mpq_stream_probe(src_dev.data_ptr(), n, None, _stream_ptr(stream)), "mpq_stream_probe")


def raw_status(name: str, *args) -> int:
    """Call an entry point with raw integers/pointers and return its status (used by error-path tests)."""
    return int(getattr(lib(), name)(*args))
