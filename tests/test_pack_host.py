"""Host-side logic of the library (no GPU): the shared object loads and exports every declared
symbol, the packer round-trips through an independent reader, validation rejects malformed input,
and the average-bit function reproduces the paper's printed values."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import mpq_synth as synth
import paper_2311_16442_amd as mpq
import unpack as up

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "mpq.h")).read()
    declared = sorted(set(re.findall(r"\b(mpq_[a-z_0-9]+)\s*\(", text)))
    assert set(declared) == set(mpq.EXPORTS)
    L = mpq.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert mpq.status_str(0) == "ok" and mpq.status_str(5).startswith("outlier")


def test_library_exports_no_other_function():
    """Nothing but the calls that mpq.h declares is a global function of the shared object (the kernels' weak
    handles, which the HIP runtime registers, are not functions a caller could link against)."""
    import shutil
    import subprocess
    if not shutil.which("nm"):
        pytest.skip("nm not available")
    out = subprocess.run(["nm", "-D", "--defined-only", mpq.LIB_PATH], check=True, capture_output=True, text=True).stdout
    functions = sorted(line.split()[2] for line in out.splitlines() if len(line.split()) == 3 and line.split()[1] == "T")
    assert functions == sorted(mpq.EXPORTS)


def test_timeline_build_adds_only_its_buffer_call():
    """The timeline build is the product sources plus phase stamps: the same exports and mpq_timeline_buffer."""
    import ctypes
    path = os.path.join(os.path.dirname(mpq.LIB_PATH), "libmpq_timeline.so")
    if not os.path.exists(path):
        pytest.skip("timeline library not built")
    L = ctypes.CDLL(path)
    for name in list(mpq.EXPORTS) + ["mpq_timeline_buffer"]:
        assert hasattr(L, name), name
    assert not hasattr(mpq.lib(), "mpq_timeline_buffer")


CASES = [
    # N, K, g1, g2, f4, p_o, z1_full, g2_axis
    (48, 1024, 64, 16, 0.10, 0.005, False, 0),
    (37, 704, 64, 4, 0.30, 0.02, True, 0),      # ragged: N % 16 != 0, G = 11, S = 3 with a short tail
    (20, 1024, 128, 2, 0.25, 0.01, True, 0),    # g1 = 128
    (16, 512, 64, 16, 0.0, 0.01, False, 0),     # no 4-bit group
    (16, 512, 64, 16, 1.0, 0.0, False, 0),      # only 4-bit groups
    (5, 64, 64, 1, 0.0, 0.2, False, 0),         # a single group
    (40, 512, 16, 16, 0.25, 0.01, True, 1),     # the paper's operating point: g1 = g2 = 16, pairs shared by 16 rows
    (40, 432, 16, 4, 0.26, 0.02, True, 1),      # 27 groups: 20 two-bit (5 units), 7 four-bit (3.5 units); 4 blocks of rows per tile
    (70, 480, 32, 32, 0.20, 0.01, True, 1),     # g1 = 32; a pair spans two tiles
    (33, 480, 32, 3, 0.20, 0.01, False, 0),     # g1 = 32 with pairs along K
    (24, 320, 16, 16, 0.0, 0.05, False, 0),     # g1 = 16, only 2-bit groups
    (24, 1024, 64, 8, 0.10, 0.005, False, 1),   # one piece per unit, pairs shared by 8 rows
    # the paper's aligned metadata (Sec. 3.3): 16-bit word per three 2-bit groups, byte per 4-bit group, byte-padded z2
    (40, 512, 16, 16, 0.25, 0.01, False, 1, 1),   # 24 two-bit groups = 8 triples, 8 four-bit groups
    (37, 432, 16, 4, 0.26, 0.02, False, 1, 1),    # 20 two-bit groups: last triple holds two; ragged rows; 4 blocks of rows per tile
    (24, 320, 16, 16, 0.0, 0.05, False, 0, 1),    # pairs along K, no 4-bit group
    (20, 256, 16, 32, 1.0, 0.0, False, 1, 1),     # only 4-bit groups, a pair spans two tiles
]


@pytest.mark.parametrize("case", CASES)
def test_pack_round_trips_through_independent_reader(case):
    N, K, g1, g2, f4, p_o, z1_full, axis = case[:8]
    meta = case[8] if len(case) > 8 else 0
    lg = synth.make_matrix(synth.MatrixSpec("t", N, K, g1, g2, f4, p_o, 77 + N + K, axis, meta), z1_full_range=z1_full)
    pk = mpq.pack_logical(lg)
    assert pk.blob.size == mpq.packed_size(N, K, g1, g2, lg.is4, lg.row_ptr, axis, meta)
    info = mpq.blob_info(pk.header)
    assert (info["N"], info["K"], info["g1"], info["g2"], info["nnz"], info["n4"], info["meta"]) == \
        (N, K, g1, g2, lg.nnz, int(lg.is4.sum()), meta)
    assert info["total_bytes"] == pk.blob.size
    u = up.unpack(pk.blob)
    assert np.array_equal(u["is4"], lg.is4)
    for name in ("codes", "s_int", "z1", "s2", "z2", "row_ptr", "col", "val"):
        assert np.array_equal(u[name], getattr(lg, name)), name
    assert not u["pad_rows_codes"].any() and not u["pad_s"].any()
    # every section offset is 256-byte aligned, every unit 16-byte aligned
    assert u["h"]["off_units"] % 256 == 0 and u["h"]["off_tiles"] % 256 == 0
    # padding overhead of the layout stays small next to the algorithmic bytes
    algo = synth.stored_bytes(lg.spec, int(lg.is4.sum()), lg.nnz)["total"]
    if N % 16 == 0 and N * K >= 16 * 1024:
        assert pk.blob.size <= algo * 1.25 + 4096


def test_pack_is_deterministic_and_position_independent():
    lg = synth.make_matrix(synth.MatrixSpec("t", 32, 512, 64, 16, 0.25, 0.01, 5))
    a = mpq.pack_logical(lg).blob
    b = mpq.pack_logical(lg).blob
    assert np.array_equal(a, b)


def _ptrs(lg):
    return dict(N=lg.spec.N, K=lg.spec.K, g1=lg.spec.g1, g2=lg.spec.g2, is4=lg.is4, codes=lg.codes,
                s_int=lg.s_int, z1=lg.z1, s2=lg.s2, z2=lg.z2, row_ptr=lg.row_ptr, col=lg.col, val=lg.val)


def _status(**kw):
    try:
        mpq.pack(**kw)
    except mpq.MpqError as e:
        return e.status
    return mpq.MPQ_OK


def test_pack_rejects_malformed_input():
    lg = synth.make_matrix(synth.MatrixSpec("t", 32, 512, 64, 4, 0.25, 0.05, 6))
    base = _ptrs(lg)
    assert _status(**base) == mpq.MPQ_OK
    g2bit = int(np.nonzero(lg.is4 == 0)[0][0])
    g4bit = int(np.nonzero(lg.is4)[0][0])
    bad = dict(base); bad["codes"] = lg.codes.copy(); bad["codes"][3, g2bit * 64 + 5] = 4
    assert _status(**bad) == mpq.MPQ_ERR_CODE_RANGE
    bad = dict(base); bad["codes"] = lg.codes.copy(); bad["codes"][3, g4bit * 64 + 5] = 16
    assert _status(**bad) == mpq.MPQ_ERR_CODE_RANGE
    r = int(np.nonzero(np.diff(lg.row_ptr) > 1)[0][0])
    e = int(lg.row_ptr[r])
    bad = dict(base); bad["col"] = lg.col.copy(); bad["col"][e + 1] = bad["col"][e]
    assert _status(**bad) == mpq.MPQ_ERR_CSR                      # not strictly increasing
    bad = dict(base); bad["col"] = lg.col.copy(); bad["col"][lg.row_ptr[r + 1] - 1] = g4bit * 64 + 63 if g4bit * 64 + 63 > lg.col[lg.row_ptr[r + 1] - 2] else 0
    assert _status(**bad) in (mpq.MPQ_ERR_OUTLIER_IN_4BIT, mpq.MPQ_ERR_CSR)
    bad = dict(base); bad["row_ptr"] = lg.row_ptr.copy(); bad["row_ptr"][4] = bad["row_ptr"][3] - 1
    assert _status(**bad) == mpq.MPQ_ERR_CSR
    bad = dict(base); bad["row_ptr"] = lg.row_ptr.copy(); bad["row_ptr"][0] = 1
    assert _status(**bad) == mpq.MPQ_ERR_CSR
    bad = dict(base); bad["col"] = lg.col.copy(); bad["col"][e] = 600
    assert _status(**bad) == mpq.MPQ_ERR_CSR                      # col >= K
    assert _status(**dict(base, K=500)) == mpq.MPQ_ERR_SHAPE      # K % g1 != 0
    assert _status(**dict(base, g1=8)) == mpq.MPQ_ERR_UNSUPPORTED       # a piece shorter than a decode step
    assert _status(**dict(base, g2_axis=1, g2=3)) == mpq.MPQ_ERR_UNSUPPORTED   # blocks of 3 rows straddle tiles
    assert _status(**dict(base, g2_axis=2)) == mpq.MPQ_ERR_SHAPE
    assert _status(**dict(base, g2=0)) == mpq.MPQ_ERR_SHAPE


def test_outlier_in_4bit_group_is_its_own_error():
    lg = synth.make_matrix(synth.MatrixSpec("t", 16, 256, 64, 4, 0.25, 0.0, 8))
    g4bit = int(np.nonzero(lg.is4)[0][0])
    rp = np.zeros(17, np.int32); rp[1:] = 1
    st = _status(**dict(_ptrs(lg), row_ptr=rp, col=np.array([g4bit * 64 + 1], np.uint16),
                        val=np.array([0x3C00], np.uint16)))
    assert st == mpq.MPQ_ERR_OUTLIER_IN_4BIT


def test_small_buffer_and_bad_header_are_reported():
    lg = synth.make_matrix(synth.MatrixSpec("t", 16, 256, 64, 4, 0.25, 0.01, 9))
    pk = mpq.pack_logical(lg)
    L = mpq.lib()
    d = mpq.Desc(16, 256, 64, 4, 0)
    arrs = [np.ascontiguousarray(a) for a in (lg.is4, lg.codes, lg.s_int, lg.z1, lg.s2, lg.z2, lg.row_ptr, lg.col, lg.val)]
    ptrs = mpq.LogicalPtrs(*[a.ctypes.data for a in arrs])
    small = np.zeros(pk.blob.size - 1, np.uint8)
    assert L.mpq_pack_host(C.byref(d), C.byref(ptrs), small.ctypes.data_as(C.c_void_p), small.size) == mpq.MPQ_ERR_SIZE
    assert L.mpq_pack_host(None, C.byref(ptrs), small.ctypes.data_as(C.c_void_p), small.size) == mpq.MPQ_ERR_NULL
    hdr = pk.header.copy(); hdr[0] ^= 0xFF
    with pytest.raises(mpq.MpqError) as ei:
        mpq.blob_info(hdr)
    assert ei.value.status == mpq.MPQ_ERR_BLOB
    # device entry points validate the header on the host before touching the GPU
    hdr = pk.header.copy(); hdr[8] ^= 1          # N changed: recorded offsets no longer match
    fake = C.c_void_p(4096)
    assert L.mpq_gemv(hdr.ctypes.data_as(C.c_void_p), fake, fake, fake, None) == mpq.MPQ_ERR_BLOB
    assert L.mpq_gemv(pk.header.ctypes.data_as(C.c_void_p), None, fake, fake, None) == mpq.MPQ_ERR_NULL
    assert L.mpq_gemv(pk.header.ctypes.data_as(C.c_void_p), C.c_void_p(4100), fake, fake, None) == mpq.MPQ_ERR_ALIGN
    assert L.mpq_gemm(pk.header.ctypes.data_as(C.c_void_p), fake, fake, fake, 0, None, 0, None) == mpq.MPQ_ERR_SHAPE
    assert L.mpq_gemm(pk.header.ctypes.data_as(C.c_void_p), fake, fake, fake, 33, None, 0, None) == mpq.MPQ_ERR_SHAPE
    assert L.mpq_dequant(pk.header.ctypes.data_as(C.c_void_p), fake, None, 0, None) == mpq.MPQ_ERR_NULL


def test_avg_bits_reproduces_the_papers_values():
    # Sec. 3.3 formula at the paper's operating point (g1 = g2 = 16, Ns = 4, 25 % / 10 % 4-bit)
    assert abs(mpq.avg_bits(1024, 1024, 16, 16, n4=16, nnz=0, mode=1, ns_bits=4) - 2.83984375) < 1e-12
    v10 = mpq.avg_bits(1280, 1280, 16, 16, n4=8, nnz=0, mode=1, ns_bits=4)
    assert abs(v10 - 2.6078125) < 1e-12
    # Sec. 4.2: 1.5 % outliers cost 0.45 bit
    with_o = mpq.avg_bits(1000, 1600, 16, 16, n4=25, nnz=24000, mode=1, ns_bits=4)
    assert abs(with_o - mpq.avg_bits(1000, 1600, 16, 16, n4=25, nnz=0, mode=1, ns_bits=4) - 0.45) < 1e-12
    # stored bits: the benchmark's headline layer is about 2.62 bits per weight
    spec = synth.config_specs(1)[1]
    nnz = int(round(spec.p_o * spec.N * (spec.G - spec.n4) * spec.g1))
    by = synth.stored_bytes(spec, spec.n4, nnz)["total"]
    got = mpq.avg_bits(spec.N, spec.K, spec.g1, spec.g2, spec.n4, nnz, mode=0)
    assert abs(got - 8.0 * by / (spec.N * spec.K)) < 1e-9 and abs(got - 2.62) < 0.01
    assert mpq.avg_bits(0, 1024, 64, 16, 0, 0) < 0


def test_group_count_beyond_the_table_offsets_is_unsupported():
    # the unit table addresses a group's scale entries with 16-bit byte offsets: 32 * G <= 65535
    rp = np.zeros(17, dtype=np.int32)
    assert mpq.packed_size(16, 2047 * 16, 16, 16, np.zeros(2047, np.uint8), rp, 1) > 0
    with pytest.raises(mpq.MpqError) as e:
        mpq.packed_size(16, 2049 * 16, 16, 16, np.zeros(2049, np.uint8), rp, 1)
    assert e.value.status == mpq.MPQ_ERR_UNSUPPORTED
    # pairs shared by single rows: 16 entries per group and tile, so the limit comes earlier
    with pytest.raises(mpq.MpqError) as e:
        mpq.packed_size(16, 1100 * 16, 16, 1, np.zeros(1100, np.uint8), rp, 1)
    assert e.value.status == mpq.MPQ_ERR_UNSUPPORTED
    assert mpq.packed_size(16, 1000 * 16, 16, 1, np.zeros(1000, np.uint8), rp, 1) > 0


def test_gemm_workspace_size_validates_before_it_asks_the_device():
    # the size depends on the compute-unit count of the current device, which the call queries: without
    # a device a valid query fails with MPQ_ERR_HIP (never a guessed size); bad arguments are refused
    # before the device is asked, so these checks need no GPU.  With a device the sizes are positive,
    # grow with the batch and hold at least one range of partial sums plus the transposed activations.
    spec = synth.MatrixSpec("ws", 4096, 4096, 64, 16, 0.10, 0.005, 77)
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    L = mpq.lib()
    n = C.c_size_t(0)
    hp = pk.header.ctypes.data_as(C.c_void_p)
    assert L.mpq_gemm_workspace_size(hp, 0, C.byref(n)) == mpq.MPQ_ERR_SHAPE
    assert L.mpq_gemm_workspace_size(hp, 33, C.byref(n)) == mpq.MPQ_ERR_SHAPE
    assert L.mpq_gemm_workspace_size(None, 4, C.byref(n)) == mpq.MPQ_ERR_NULL
    assert L.mpq_gemm_workspace_size(hp, 4, None) == mpq.MPQ_ERR_NULL
    bad = pk.header.copy()
    bad[8] ^= 1
    assert L.mpq_gemm_workspace_size(bad.ctypes.data_as(C.c_void_p), 4, C.byref(n)) == mpq.MPQ_ERR_BLOB
    st = L.mpq_gemm_workspace_size(hp, 4, C.byref(n))
    assert st in (mpq.MPQ_OK, mpq.MPQ_ERR_HIP)
    if st == mpq.MPQ_OK:
        assert mpq.gemm_workspace_size(pk.header, 1) == 0
        sizes = [mpq.gemm_workspace_size(pk.header, M) for M in (2, 8, 9, 16, 17, 32)]
        assert all(b > 0 for b in sizes) and sizes == sorted(sizes)
        assert sizes[0] >= (4096 // 16) * 16 * 16 * 4 + 4096 * 8 * 2
        assert mpq.gemm_workspace_size_planned(pk.header, 8, mpq.Plan(lb_min_ranges=3)) > sizes[1]


def test_avg_bits_with_the_papers_aligned_metadata_stays_within_its_stated_overhead():
    # Sec. 3.3: packing the metadata as the paper describes changes the average by less than 0.02 bit
    # at its operating point (g1 = g2 = 16, Ns = 4, 25 % 4-bit): 16 bits per three groups instead of
    # 3 x (2 + 4), an 8-bit padded second-order zero instead of 4 bits
    spec = dict(N=4096, K=4096, g1=16, g2=16, g2_axis=1)
    G = 4096 // 16
    ideal = mpq.avg_bits(n4=G // 4, nnz=0, mode=1, ns_bits=4, **spec)
    aligned = mpq.avg_bits(n4=G // 4, nnz=0, mode=2, ns_bits=4, **spec)
    assert abs(ideal - 2.84) < 0.005
    assert abs(aligned - (0.75 * (2 + 16 / 48 + 24 / 256) + 1.0)) < 1e-12
    assert abs(aligned - ideal) < 0.02
    assert mpq.avg_bits(n4=0, nnz=0, mode=3, ns_bits=4, **spec) < 0
