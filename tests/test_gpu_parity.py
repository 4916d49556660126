"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Dequantized weights must be bit-exact; products must stay within 2e-3 of the
oracle's binary64 accumulation (relative, with the small-output floor of gpu_util.rel_err)."""
import numpy as np
import pytest

import mpq_synth as synth
import oracle
import paper_2311_16442_amd as mpq
from gpu_util import Guarded, Workspace, rel_err, to_dev

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    return t


CASES = [
    # name, N, K, g1, g2, f4, p_o, z1_full
    ("config0", 1024, 1024, 64, 16, 0.10, 0.005, False),
    ("ragged_rows", 1000, 704, 64, 4, 0.30, 0.02, True),     # N % 16 = 8, G = 11, S = 3 (short tail group)
    ("g128", 208, 2048, 128, 16, 0.15, 0.005, True),
    ("only_2bit", 64, 512, 64, 16, 0.0, 0.01, False),
    ("only_4bit", 64, 512, 64, 16, 1.0, 0.0, True),
    ("one_group", 5, 64, 64, 1, 0.0, 0.2, False),
    ("down_like", 272, 11008, 64, 16, 0.10, 0.005, False),   # G = 172 = 10*16 + 12
    ("wide", 48, 28672, 64, 16, 0.10, 0.005, False),         # largest K of the configurations
    ("dense_outliers", 96, 1024, 64, 16, 0.10, 0.30, False), # rows with hundreds of outliers
    # first-order groups shorter than a 16-byte unit and second-order pairs shared by rows (last field:
    # 1 = a pair covers the same K-group of g2 rows, the paper's axis, Sec. 2.2)
    ("paper_point", 1000, 1024, 16, 16, 0.25, 0.005, True, 1),   # g1 = g2 = 16, 25 % 4-bit
    ("g32_rows32", 208, 2048, 32, 32, 0.15, 0.005, True, 1),     # a pair spans two tiles
    ("g16_along_k", 272, 1520, 16, 16, 0.10, 0.01, False, 0),    # 95 groups: ragged units in both streams
    ("g64_rows4", 100, 1024, 64, 4, 0.10, 0.005, True, 1),       # four blocks of rows per tile
    # the paper's aligned metadata (Sec. 3.3 "Memory Alignment"; last field 1): a 16-bit word per three 2-bit
    # groups with two 3-bit scales, a byte per 4-bit group, a byte-padded integer second-order zero
    ("aligned_paper_point", 1000, 1024, 16, 16, 0.25, 0.005, False, 1, 1),  # g1 = g2 = 16, pairs shared by 16 rows
    ("aligned_along_k", 272, 1520, 16, 4, 0.10, 0.01, False, 0, 1),         # 95 groups: a short last triple, ragged units
    ("aligned_rows4", 100, 2048, 16, 4, 0.30, 0.005, False, 1, 1),          # four blocks of rows per tile
]


def make(case):
    name, N, K, g1, g2, f4, p_o, z1_full = case[:8]
    axis = case[8] if len(case) > 8 else 0
    meta = case[9] if len(case) > 9 else 0
    lg = synth.make_matrix(synth.MatrixSpec(name, N, K, g1, g2, f4, p_o, 4242 + N + K, axis, meta), z1_full_range=z1_full)
    return lg, oracle.Matrix.from_logical(lg), mpq.pack_logical(lg)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_dequant_bit_exact(torch, case):
    lg, om, pk = make(case)
    print("case", case, flush=True)
    blob = to_dev(torch, pk.blob)
    for add in (False, True):
        out = Guarded(torch, pk.N * pk.K)
        mpq.dequant(pk.header, blob, out.view, add_outliers=add)
        got = out.check_and_get().reshape(pk.N, pk.K)
        ref = om.dequant(add)
        bad = np.argwhere(got != ref)
        assert bad.size == 0, (add, bad[:5], got[tuple(bad[0])], ref[tuple(bad[0])])


def test_dequant_with_a_unit_table_too_long_to_stage(torch):
    # K = 40960: 142 blocks per tile, a unit table of 4.4 KiB, which the kernel reads from memory instead of LDS
    case = ("longest", 48, 40960, 64, 16, 0.10, 0.01, False)
    lg, om, pk = make(case)
    assert 32 * (pk.header.view(np.int32)[13] + pk.header.view(np.int32)[14]) > 4096   # B2 + B4 blocks, 32 bytes of table each
    blob = to_dev(torch, pk.blob)
    for add in (False, True):
        out = Guarded(torch, pk.N * pk.K)
        mpq.dequant(pk.header, blob, out.view, add_outliers=add)
        got = out.check_and_get().reshape(pk.N, pk.K)
        assert np.array_equal(got, om.dequant(add)), add


# Groups narrower than a 128-byte line of the output: workgroups own 16 rows x 2048 columns and decode every unit
# with a piece in them, as long as the unit table fits their LDS (14 KiB); longer rows take the per-block kernel.
NARROW_CASES = [
    ("g16_ranges", 100, 5008, 16, 16, 0.25, 0.02, True, 1),              # two ranges and a ragged third; > 32 outliers per (row, range)
    ("g16_ranges_aligned", 100, 5008, 16, 16, 0.25, 0.02, False, 1, 1),  # the same with the aligned metadata
    ("g32_ranges", 72, 6176, 32, 16, 0.10, 0.02, True, 0),
    ("g16_mostly_4bit", 40, 4112, 16, 16, 0.97, 0.01, False, 1),         # 17 passes of 4-bit units in a range: a second batch
    ("g16_no_4bit", 24, 4096, 16, 16, 0.0, 0.01, False, 0),
    ("g16_long", 32, 24576, 16, 16, 0.25, 0.01, False, 1),               # unit table of 15 KiB: per-block kernel, table in LDS
    ("g16_long_aligned", 32, 24576, 16, 16, 0.25, 0.01, False, 1, 1),
    ("g32_longest", 16, 65504, 32, 16, 0.10, 0.005, False, 0),           # 21 KiB: per-block kernel, table read from memory
    ("g16_only_4bit", 40, 2064, 16, 16, 1.0, 0.0, False, 1),             # no 2-bit stream at all
]


@pytest.mark.parametrize("case", NARROW_CASES, ids=[c[0] for c in NARROW_CASES])
def test_dequant_of_narrow_groups(torch, case):
    lg, om, pk = make(case)
    print("case", case, flush=True)
    hdr = pk.header.view(np.int32)
    table = 32 * (64 // case[3]) * (hdr[13] + hdr[14])   # bytes per block of the table x (B2 + B4)
    assert (table > 14336) == ("long" in case[0]), table
    blob = to_dev(torch, pk.blob)
    for add in (False, True):
        out = Guarded(torch, pk.N * pk.K)
        mpq.dequant(pk.header, blob, out.view, add_outliers=add)
        got = out.check_and_get().reshape(pk.N, pk.K)
        ref = om.dequant(add)
        bad = np.argwhere(got != ref)
        assert bad.size == 0, (add, bad[:5], got[tuple(bad[0])], ref[tuple(bad[0])])


def test_dequant_of_seeded_random_shapes(torch):
    # 40 shapes drawn from a fixed seed: group widths, both axes and packings, group counts around the 2048-column
    # ranges of the whole-line kernel (127 .. 130, 256, 257 groups of 16), rows from 1 to 100, 4-bit shares from 0 to 1
    rng = np.random.default_rng(20231116)
    for c in range(40):
        g1 = int(rng.choice([16, 16, 32, 32, 64]))
        meta = int(rng.integers(0, 2)) if g1 == 16 else 0
        axis = int(rng.integers(0, 2))
        g2 = int(rng.choice([4, 16] if axis == 1 else [1, 2, 4, 16]))
        G = int(rng.choice([1, 2, 3, 5, 64, 127, 128, 129, 130, 200, 256, 257, 300, 384, 400, 512, 640]))
        G = min(G, 160) if g1 == 64 else G
        N = int(rng.choice([1, 5, 16, 17, 31, 32, 48, 100]))
        f4 = float(rng.choice([0.0, 0.05, 0.25, 0.5, 0.9, 1.0]))
        p_o = float(rng.choice([0.0, 0.005, 0.02, 0.1]))
        case = (f"r{c}", N, G * g1, g1, g2, f4, p_o, False, axis, meta)
        print("case", case, flush=True)
        lg, om, pk = make(case)
        blob = to_dev(torch, pk.blob)
        for add in (False, True):
            out = Guarded(torch, pk.N * pk.K)
            mpq.dequant(pk.header, blob, out.view, add_outliers=add)
            assert np.array_equal(out.check_and_get().reshape(pk.N, pk.K), om.dequant(add)), (case, add)


@pytest.mark.parametrize("case", [("beyond_index", 16, 8192, 64, 16, 0.0, 0.6, False),
                                  ("g16_beyond_index", 16, 8192, 16, 16, 0.1, 0.65, False, 1)], ids=["g64", "g16"])
def test_dequant_of_a_tile_with_more_outliers_than_its_block_index_can_count(torch, case):
    # more than 65535 outliers in one 16-row tile: the blob carries no outlier block index (16-bit entries), and the
    # outliers are added to the finished matrix by a second kernel
    lg, om, pk = make(case)
    assert lg.row_ptr[-1] > 65535 and pk.header.view(np.uint64)[16] == 0   # oidx_off
    blob = to_dev(torch, pk.blob)
    for add in (False, True):
        out = Guarded(torch, pk.N * pk.K)
        mpq.dequant(pk.header, blob, out.view, add_outliers=add)
        assert np.array_equal(out.check_and_get().reshape(pk.N, pk.K), om.dequant(add)), add


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_gemv_within_tolerance(torch, case):
    lg, om, pk = make(case)
    print("case", case, flush=True)
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(99, 1, pk.K)
    x = to_dev(torch, X[0].view(np.int16))
    y = Guarded(torch, pk.N)
    mpq.gemv(pk.header, blob, x, y.view)
    got = y.check_and_get()
    ref = om.gemm(X, threads=8)[0]
    e_floor, e_max = rel_err(got, ref)
    assert e_floor <= TOL, (e_floor, e_max)
    # a second launch gives the same bits (fixed reduction order, no races)
    y2 = Guarded(torch, pk.N)
    mpq.gemv(pk.header, blob, x, y2.view)
    assert np.array_equal(y2.check_and_get(), got)


def test_products_of_seeded_random_shapes(torch):
    # 30 shapes drawn from a fixed seed, each at M = 1 and two batch sizes from 2 to 32: every group width, both axes
    # and packings, 1 to 4096 rows, K from one group to 25600 columns, 4-bit shares from 0 to 1
    rng = np.random.default_rng(2311_16442)
    worst = 0.0
    for c in range(30):
        g1 = int(rng.choice([16, 32, 64, 64, 128]))
        meta = int(rng.integers(0, 2)) if g1 == 16 else 0
        axis = int(rng.integers(0, 2))
        g2 = int(rng.choice([4, 16] if axis == 1 else [1, 2, 4, 16]))
        G = int(rng.choice([1, 2, 3, 5, 16, 31, 64, 65, 100, 128, 172, 200]))
        N = int(rng.choice([1, 5, 16, 17, 48, 100, 256, 1000, 4096]))
        N = 256 if N * G * g1 > 40e6 else N
        f4 = float(rng.choice([0.0, 0.1, 0.25, 0.5, 1.0]))
        p_o = float(rng.choice([0.0, 0.005, 0.015]))
        Ms = [1] + [int(m) for m in rng.choice([2, 3, 4, 7, 8, 9, 12, 16, 17, 24, 31, 32], size=2, replace=False)]
        case = (f"r{c}", N, G * g1, g1, g2, f4, p_o, False, axis, meta)
        print("case", case, Ms, flush=True)
        lg, om, pk = make(case)
        blob = to_dev(torch, pk.blob)
        for M in Ms:
            X = synth.make_x(77 + c + M, M, pk.K)
            Y = Guarded(torch, M * pk.N)
            if M == 1:
                mpq.gemv(pk.header, blob, to_dev(torch, X[0].view(np.int16)), Y.view)
            else:
                ws = Workspace(torch, mpq, pk.header, M)
                mpq.gemm(pk.header, blob, to_dev(torch, X.view(np.int16)), Y.view, M, workspace=ws.view)
                ws.check()
            e_floor, e_max = rel_err(Y.check_and_get().reshape(M, pk.N), om.gemm(X, threads=8))
            worst = max(worst, e_floor)
            assert e_floor <= TOL, (case, M, e_floor, e_max)
    print("worst error", worst)


def test_gemv_exact_for_integer_problem(torch):
    # identity scales and small integer activations: y = codes @ x in integers, exactly representable
    lg = synth.make_matrix(synth.MatrixSpec("int", 64, 256, 64, 2, 0.25, 0.0, 31))
    lg.s_int[:] = 1; lg.z1[:] = 0; lg.s2[:] = 0x3C00; lg.z2[:] = 0
    pk = mpq.pack_logical(lg)
    rng = np.random.default_rng(32)
    xi = rng.integers(-1, 2, size=256)
    ref = lg.codes.astype(np.int64) @ xi
    assert np.max(np.abs(ref)) < 2048
    y = Guarded(torch, 64)
    mpq.gemv(pk.header, to_dev(torch, pk.blob), to_dev(torch, xi.astype(np.float16).view(np.int16)), y.view)
    assert np.array_equal(y.check_and_get().view(np.float16).astype(np.int64), ref)


def test_special_scale_values_bit_exact(torch):
    # any uint8 s_int / z1 and any finite fp16 pair must decode: negative scales, results that are
    # subnormal, zero with either sign, or overflow to infinity
    N, K, g1, g2 = 64, 1024, 64, 1
    lg = synth.make_matrix(synth.MatrixSpec("edge", N, K, g1, g2, 0.25, 0.01, 33), z1_full_range=True)
    rng = np.random.default_rng(34)
    specials = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF, 0x3C00, 0xBC00,
                         0x0200, 0x1400, 0x5BF8, 0x57F8, 0x4248, 0x2E66], dtype=np.uint16)
    lg.s2[:] = rng.choice(specials, size=lg.s2.shape)
    lg.z2[:] = rng.choice(specials, size=lg.z2.shape)
    lg.s_int[:, :4] = np.array([0, 1, 254, 255], dtype=np.uint8)
    om, pk = oracle.Matrix.from_logical(lg), mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    for add in (False, True):
        out = Guarded(torch, N * K)
        mpq.dequant(pk.header, blob, out.view, add_outliers=add)
        got, ref = out.check_and_get().reshape(N, K), om.dequant(add)
        nan = (ref & 0x7FFF) > 0x7C00
        assert np.array_equal((got & 0x7FFF) > 0x7C00, nan)       # NaN (inf - inf, 0 * inf) where the oracle has NaN
        assert np.array_equal(got[~nan], ref[~nan])
        kinds = ref[~nan] & 0x7FFF
        assert (kinds == 0x7C00).any() and ((kinds > 0) & (kinds < 0x0400)).any() and (kinds == 0).any()


def test_padding_bytes_are_never_used(torch):
    import unpack as up
    lg = synth.make_matrix(synth.MatrixSpec("pad", 40, 704, 64, 4, 0.30, 0.02, 35))
    om, pk = oracle.Matrix.from_logical(lg), mpq.pack_logical(lg)
    h = up.read_header(pk.blob)
    poisoned = pk.blob.copy()
    # padding units of both streams (unit index >= U2 / U4) in every tile
    C = h["B2"] + h["B4"]
    tiles = poisoned[h["off_tiles"]: h["off_tiles"] + h["T"] * h["tile_stride"]].reshape(h["T"], h["tile_stride"])
    npad = 0
    for u in list(range(h["U2"], 4 * h["B2"])) + list(range(4 * h["B2"] + h["U4"], 4 * C)):
        at = h["codes_off"] + (u // 4) * 1024 + (u % 4) * 256      # 16 rows x 16 bytes of unit u
        tiles[:, at: at + 256] = 0xFF
        npad += 1
    assert npad > 0 and np.count_nonzero(poisoned != pk.blob) > 0
    blob = to_dev(torch, poisoned)
    X = synth.make_x(36, 1, 704)
    y = Guarded(torch, 40)
    mpq.gemv(pk.header, blob, to_dev(torch, X[0].view(np.int16)), y.view)
    assert rel_err(y.check_and_get(), om.gemm(X)[0])[0] <= TOL
    out = Guarded(torch, 40 * 704)
    mpq.dequant(pk.header, blob, out.view, add_outliers=True)
    assert np.array_equal(out.check_and_get().reshape(40, 704), om.dequant(True))


@pytest.mark.parametrize("M", [1, 2, 4, 8, 16, 32])
def test_gemm_within_tolerance(torch, M):
    lg, om, pk = make(CASES[1])
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(123 + M, M, pk.K)
    Y = Guarded(torch, M * pk.N)
    ws = Workspace(torch, mpq, pk.header, M)
    mpq.gemm(pk.header, blob, to_dev(torch, X.view(np.int16)), Y.view, M, workspace=ws.view)
    got = Y.check_and_get().reshape(M, pk.N)
    ws.check()
    ref = om.gemm(X, threads=8)
    e_floor, e_max = rel_err(got, ref)
    assert e_floor <= TOL, (M, e_floor, e_max)


def test_outliers_reduce_to_csr_product(torch):
    import scipy.sparse as sp
    lg = synth.make_matrix(synth.MatrixSpec("csr", 160, 1024, 64, 16, 0.10, 0.02, 37))
    lg.codes[:] = np.repeat(lg.z1, 64, axis=1)      # dense part decodes to zero
    pk = mpq.pack_logical(lg)
    X = synth.make_x(38, 1, 1024)
    y = Guarded(torch, 160)
    mpq.gemv(pk.header, to_dev(torch, pk.blob), to_dev(torch, X[0].view(np.int16)), y.view)
    A = sp.csr_matrix((lg.val.view(np.float16).astype(np.float64), lg.col.astype(np.int64),
                       lg.row_ptr.astype(np.int64)), shape=(160, 1024))
    ref = A @ X[0].view(np.float16).astype(np.float64)
    assert rel_err(y.check_and_get(), ref)[0] <= TOL


@pytest.mark.parametrize("path", [mpq.KERNEL_GEMV_PLANES, mpq.KERNEL_GEMV_DECODE])
@pytest.mark.parametrize("waves,tiles", [(8, 1), (8, 2), (8, 3), (16, 1), (16, 2), (16, 5), (8, 8)])
def test_gemv_work_splits_agree_with_oracle(torch, waves, tiles, path):
    # every work split of both matrix-vector kernels (waves per workgroup x tiles per workgroup, forced
    # through a launch plan) on a ragged shape: 63 tiles, last one with 8 rows, a short tail
    # super-group, fewer code blocks per tile (6) than waves
    lg, om, pk = make(("ragged_rows", 1000, 704, 64, 4, 0.30, 0.02, True))
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(7, 1, pk.K)
    x = to_dev(torch, X[0].view(np.int16))
    ref = om.gemm(X, threads=8)[0]
    plan = mpq.Plan(gemv_path=path, gemv_waves=waves, gemv_tiles=tiles)
    print("path", path, "waves", waves, "tiles", tiles, flush=True)
    y = Guarded(torch, pk.N)
    rep = mpq.gemm_planned(pk.header, blob, x, y.view, 1, plan=plan)
    got = y.check_and_get()
    assert (rep.kernel, rep.waves, rep.tiles_per_workgroup, rep.launches) == (path, waves, tiles, 1)
    e_floor, e_max = rel_err(got, ref)
    assert e_floor <= TOL, (e_floor, e_max)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_both_gemv_kernels_on_every_case(torch, case):
    # the plane-sum kernel (2-bit groups through the fp8/fp4 matrix instruction) where the format allows
    # it (one group per unit: g1 >= 64), the per-weight kernel everywhere; the automatic choice on these
    # small matrices (few tiles per compute unit) is the per-weight kernel; results are the same bits
    # from call to call
    lg, om, pk = make(case)
    print("case", case, flush=True)
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(41, 1, pk.K)
    x = to_dev(torch, X[0].view(np.int16))
    ref = om.gemm(X, threads=8)[0]
    ran = []
    for path in (0, mpq.KERNEL_GEMV_PLANES, mpq.KERNEL_GEMV_DECODE):
        y = Guarded(torch, pk.N)
        try:
            rep = mpq.gemm_planned(pk.header, blob, x, y.view, 1, plan=mpq.Plan(gemv_path=path))
        except mpq.MpqError as e:
            # groups shorter than a unit, or rows so long that the split activations do not fit on chip
            # groups shorter than a unit
            assert path == mpq.KERNEL_GEMV_PLANES and e.status == mpq.MPQ_ERR_UNSUPPORTED and pk.g1 < 64
            continue
        got = y.check_and_get()
        e_floor, e_max = rel_err(got, ref)
        assert e_floor <= TOL, (path, e_floor, e_max)
        y2 = Guarded(torch, pk.N)
        mpq.gemm_planned(pk.header, blob, x, y2.view, 1, plan=mpq.Plan(gemv_path=path))
        assert np.array_equal(y2.check_and_get(), got)
        ran.append((path, rep.kernel))
    planes_ran = (mpq.KERNEL_GEMV_PLANES, mpq.KERNEL_GEMV_PLANES) in ran
    assert planes_ran == (pk.g1 >= 64), ran      # also K = 28672, where only the fp8 pieces of the activations are on chip
    assert ran[0][1] == mpq.KERNEL_GEMV_DECODE, ran
    assert (mpq.KERNEL_GEMV_DECODE, mpq.KERNEL_GEMV_DECODE) in ran


def test_plane_sum_kernel_with_wide_ranging_activations(torch):
    # activations spanning many binades inside one 64-column unit, zeros, subnormals and the largest
    # finite fp16 values: the split into fp8 pieces is exact over this range
    name, N, K, g1, g2, f4, p_o, z1_full = CASES[0]
    lg = synth.make_matrix(synth.MatrixSpec(name, N, K, g1, g2, f4, p_o, 4242 + N + K))
    lg.s2[:] = synth.f16_bits(np.full(lg.s2.shape, 2.0e-5))     # small weights: the outputs stay inside fp16
    lg.val[:] = synth.f16_bits(lg.val.view(np.float16).astype(np.float64) * 1e-2)
    om, pk = oracle.Matrix.from_logical(lg), mpq.pack_logical(lg)
    rng = np.random.default_rng(43)
    xf = rng.normal(0.0, 1.0, size=pk.K) * np.exp2(rng.integers(-14, 6, size=pk.K))
    xf[::17] = 0.0
    xf[5::64] = 6.0e-8
    xf[9::128] = 65504.0 * np.sign(rng.normal(size=xf[9::128].size))
    X = synth.f16_bits(xf)[None, :]
    blob = to_dev(torch, pk.blob)
    y = Guarded(torch, pk.N)
    rep = mpq.gemm_planned(pk.header, blob, to_dev(torch, X[0].view(np.int16)), y.view, 1,
                           plan=mpq.Plan(gemv_path=mpq.KERNEL_GEMV_PLANES))
    assert rep.kernel == mpq.KERNEL_GEMV_PLANES
    ref = om.gemm(X, threads=8)[0]
    e_floor, e_max = rel_err(y.check_and_get(), ref)
    assert e_floor <= TOL, (e_floor, e_max)


@pytest.mark.parametrize("M", [2, 5, 16, 32])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_gemm_on_every_case(torch, case, M):
    # the batch product the library chooses by itself, on every format of the parity set
    lg, om, pk = make(case)
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(300 + M, M, pk.K)
    Y = Guarded(torch, M * pk.N)
    ws = Workspace(torch, mpq, pk.header, M)
    mpq.gemm(pk.header, blob, to_dev(torch, X.view(np.int16)), Y.view, M, workspace=ws.view)
    got = Y.check_and_get().reshape(M, pk.N)
    ws.check()
    e_floor, e_max = rel_err(got, om.gemm(X, threads=8))
    assert e_floor <= TOL, (M, e_floor, e_max)


@pytest.mark.parametrize("min_h", [0, 3])
@pytest.mark.parametrize("M", [2, 7, 8, 9, 16, 17, 32])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_large_batch_kernel_within_tolerance(torch, case, M, min_h):
    # the kernel that keeps one K-range of the activations resident per workgroup and writes partial
    # sums that a second kernel adds up, forced for every batch size through a launch plan (by
    # itself the library takes it where the other batch kernel would decode the weights several
    # times); also with at least three ranges on matrices whose activations would fit at once.  The
    # workspace has exactly the size the library asks for under the same plan, with a guard band behind it.
    lg, om, pk = make(case)
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(700 + M, M, pk.K)
    ref = om.gemm(X, threads=8)
    print("case", case, "M", M, "min_h", min_h, flush=True)
    plan = mpq.Plan(large_batch=1, lb_min_ranges=min_h)
    ws = Workspace(torch, mpq, pk.header, M, plan)
    assert ws.bytes > 0
    Y = Guarded(torch, M * pk.N)
    rep = mpq.gemm_planned(pk.header, blob, to_dev(torch, X.view(np.int16)), Y.view, M, plan=plan, workspace=ws.view)
    got = Y.check_and_get().reshape(M, pk.N)
    Y2 = Guarded(torch, M * pk.N)
    rep2 = mpq.gemm_planned(pk.header, blob, to_dev(torch, X.view(np.int16)), Y2.view, M, plan=plan, workspace=ws.view)
    again = Y2.check_and_get().reshape(M, pk.N)
    ws.check()
    assert rep.kernel == rep2.kernel == mpq.KERNEL_BATCH_RANGES and rep.launches == 2, "the large-batch kernel did not run"
    e_floor, e_max = rel_err(got, ref)
    assert e_floor <= TOL, (e_floor, e_max)
    assert np.array_equal(got, again)


def test_large_batch_kernel_in_a_graph_and_without_workspace(torch):
    # the library allocates nothing: with the caller's workspace the large-batch kernel can be
    # captured into a graph and every replay reproduces the eager result; without a workspace (or
    # with one that is too small) the product is computed by the other batch kernel
    lg, om, pk = make(CASES[6])
    M = 16
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(900, M, pk.K)
    Xd = to_dev(torch, X.view(np.int16))
    ref = om.gemm(X, threads=8)
    stream = torch.cuda.Stream()
    plan = mpq.Plan(large_batch=1)
    ws = Workspace(torch, mpq, pk.header, M, plan)
    Y = Guarded(torch, M * pk.N)
    torch.cuda.synchronize()
    rep = mpq.gemm_planned(pk.header, blob, Xd, Y.view, M, plan=plan, stream=stream, workspace=ws.view)
    stream.synchronize()
    assert rep.kernel == mpq.KERNEL_BATCH_RANGES
    eager = Y.check_and_get().reshape(M, pk.N)
    assert rel_err(eager, ref)[0] <= TOL
    Yg = Guarded(torch, M * pk.N)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        rep = mpq.gemm_planned(pk.header, blob, Xd, Yg.view, M, plan=plan, stream=stream, workspace=ws.view)
    assert rep.kernel == mpq.KERNEL_BATCH_RANGES
    for rep_i in range(3):
        Yg.view.zero_()
        ws.buf[:ws.bytes].fill_(0xFF)      # the workspace carries nothing from call to call
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(Yg.check_and_get().reshape(M, pk.N), eager), rep_i
    ws.check()
    for small in (None, ws.view[:ws.bytes - 256]):
        Yn = Guarded(torch, M * pk.N)
        rep = mpq.gemm_planned(pk.header, blob, Xd, Yn.view, M, plan=plan, workspace=small)
        assert rep.kernel == mpq.KERNEL_BATCH_RESIDENT      # neither of the two ran the large-batch kernel
        assert rel_err(Yn.check_and_get().reshape(M, pk.N), ref)[0] <= TOL


def test_a_pending_hip_error_of_the_caller_is_neither_reported_nor_cleared(torch):
    # the library judges its launches by the launch calls' return values and leaves the thread's last-error state alone
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipSetDevice.restype = hip.hipGetLastError.restype = hip.hipPeekAtLastError.restype = ctypes.c_int
    lg, om, pk = make(CASES[0])
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(5, 4, pk.K)
    x = to_dev(torch, X.view(np.int16))
    ws = Workspace(torch, mpq, pk.header, 4)
    y, Y, out, x1 = Guarded(torch, pk.N), Guarded(torch, 4 * pk.N), Guarded(torch, pk.N * pk.K), x[:pk.K].contiguous()
    torch.cuda.synchronize()
    hip.hipGetLastError()                                 # start from a clean state
    err = hip.hipSetDevice(9999)                          # refused on the host: no such device
    assert err != 0 and hip.hipPeekAtLastError() == err
    # (no torch call from here to the caller's own hipGetLastError: torch would find the error and raise)
    try:
        mpq.gemv(pk.header, blob, x1, y.view)             # raises on any status other than MPQ_OK
        mpq.gemm(pk.header, blob, x, Y.view, 4, workspace=ws.view)
        mpq.dequant(pk.header, blob, out.view, add_outliers=True)
    finally:
        pending, after = hip.hipGetLastError(), hip.hipGetLastError()   # the caller's own check, which clears it
    assert pending == err and after == 0                  # it was still there for the caller
    assert rel_err(y.check_and_get(), om.gemm(X[:1], threads=8)[0])[0] <= TOL
    assert rel_err(Y.check_and_get().reshape(4, pk.N), om.gemm(X, threads=8))[0] <= TOL
    assert np.array_equal(out.check_and_get().reshape(pk.N, pk.K), om.dequant(True))


def test_workspace_sizes_on_the_device(torch):
    # nothing for M = 1, partial sums for every range plus the transposed activations otherwise, growing
    # with the batch and with the number of ranges a plan asks for
    lg, om, pk = make(CASES[0])
    assert mpq.gemm_workspace_size(pk.header, 1) == 0
    sizes = [mpq.gemm_workspace_size(pk.header, M) for M in (2, 8, 9, 16, 17, 32)]
    assert all(b > 0 for b in sizes) and sizes == sorted(sizes)
    assert sizes[0] >= (pk.N // 16) * 16 * 16 * 4 + pk.K * 8 * 2
    assert mpq.gemm_workspace_size_planned(pk.header, 8, mpq.Plan(lb_min_ranges=3)) > sizes[1]


def test_several_products_in_one_launch(torch):
    # mpq_gemv_multi: independent products of different shapes (ragged rows, long rows, many outliers)
    cases = [CASES[0], CASES[1], CASES[6], CASES[8], CASES[2]]
    built = [make(c) for c in cases]
    blobs = [to_dev(torch, pk.blob) for _, _, pk in built]
    Xs = [synth.make_x(900 + p, 1, pk.K) for p, (_, _, pk) in enumerate(built)]
    xs = [to_dev(torch, X[0].view(np.int16)) for X in Xs]
    ys = [Guarded(torch, pk.N) for _, _, pk in built]
    mpq.gemv_multi([pk.header for _, _, pk in built], blobs, xs, [y.view for y in ys])
    for (lg, om, pk), X, y in zip(built, Xs, ys):
        got = y.check_and_get()
        e_floor, e_max = rel_err(got, om.gemm(X, threads=8)[0])
        assert e_floor <= TOL, (lg.spec.name, e_floor, e_max)
    # a single product through the same entry point, and the error paths that need no launch
    y1 = Guarded(torch, built[0][2].N)
    mpq.gemv_multi([built[0][2].header], blobs[:1], xs[:1], [y1.view])
    assert np.array_equal(y1.check_and_get(), ys[0].check_and_get())
    lg16, om16, pk16 = make(CASES[9])                      # g1 = 16 next to g1 = 64: no common configuration
    b16 = to_dev(torch, pk16.blob)
    x16 = to_dev(torch, synth.make_x(1, 1, pk16.K)[0].view(np.int16))
    y16 = Guarded(torch, pk16.N)
    with pytest.raises(mpq.MpqError) as e:
        mpq.gemv_multi([built[0][2].header, pk16.header], [blobs[0], b16], [xs[0], x16], [ys[0].view, y16.view])
    assert e.value.status == mpq.MPQ_ERR_UNSUPPORTED
    with pytest.raises(mpq.MpqError) as e:
        mpq.gemv_multi([built[0][2].header] * 9, blobs[:1] * 9, xs[:1] * 9, [ys[0].view] * 9)
    assert e.value.status == mpq.MPQ_ERR_SHAPE
    mpq.gemv_multi([pk16.header], [b16], [x16], [y16.view])  # and g1 = 16 on its own
    e_floor, e_max = rel_err(y16.check_and_get(), om16.gemm(synth.make_x(1, 1, pk16.K), threads=8)[0])
    assert e_floor <= TOL, (e_floor, e_max)
    # the aligned metadata: three matrices in one launch; next to byte-wide metadata there is no common configuration
    al = [make(c) for c in CASES if len(c) > 9 and c[9] == 1]
    assert len(al) == 3
    bl = [to_dev(torch, pk.blob) for _, _, pk in al]
    Xa = [synth.make_x(950 + p, 1, pk.K) for p, (_, _, pk) in enumerate(al)]
    xa = [to_dev(torch, X[0].view(np.int16)) for X in Xa]
    ya = [Guarded(torch, pk.N) for _, _, pk in al]
    mpq.gemv_multi([pk.header for _, _, pk in al], bl, xa, [y.view for y in ya])
    for (lg, om, pk), X, y in zip(al, Xa, ya):
        e_floor, e_max = rel_err(y.check_and_get(), om.gemm(X, threads=8)[0])
        assert e_floor <= TOL, (lg.spec.name, e_floor, e_max)
    with pytest.raises(mpq.MpqError) as e:
        mpq.gemv_multi([pk16.header, al[0][2].header], [b16, bl[0]], [x16, xa[0]], [y16.view, ya[0].view])
    assert e.value.status == mpq.MPQ_ERR_UNSUPPORTED


def test_quantized_float_weights_end_to_end(torch):
    # float weights -> reference quantizer (library, host) -> pack -> GEMV on the GPU: parity with the
    # oracle on the quantized matrix, and the product stays near the float product (Sec. 2.2, 3.3, 4.3)
    rng = np.random.default_rng(77)
    N, K, g1, g2 = 512, 2048, 64, 16
    W = (rng.standard_t(df=5, size=(N, K)) * 0.02).astype(np.float32)
    W[:, 5 * g1:6 * g1] *= 6.0
    q = mpq.quantize(W, g1, g2, n4=int(round(0.1 * K / g1)), p_o=0.005)
    assert q["is4"][5] == 1
    pk = mpq.pack(N, K, g1, g2, **q)
    om = oracle.Matrix(N, K, g1, g2, q["is4"], q["codes"], q["s_int"], q["z1"], q["s2"], q["z2"],
                       q["row_ptr"], q["col"], q["val"])
    X = synth.make_x(5, 1, K)
    y = Guarded(torch, N)
    mpq.gemv(pk.header, to_dev(torch, pk.blob), to_dev(torch, X[0].view(np.int16)), y.view)
    got = y.check_and_get()
    ref = om.gemm(X, threads=8)[0]
    e_floor, e_max = rel_err(got, ref)
    assert e_floor <= TOL, (e_floor, e_max)
    y_float = W.astype(np.float64) @ X[0].view(np.float16).astype(np.float64)
    rel = np.linalg.norm(got.view(np.float16).astype(np.float64) - y_float) / np.linalg.norm(y_float)
    print("relative error of the quantized product against the float product:", rel, flush=True)
    assert rel < 0.5    # 2-bit groups of 64: coarse, but the product follows the float one
