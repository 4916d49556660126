"""Pins of the CPU oracle against things other than itself (all CPU, `-m "not gpu"`).

What is used as ground truth here:
  * exact rational arithmetic with a from-first-principles rounding (tests/brute.py);
  * numpy's IEEE half type for conversions and for the per-weight operation sequence;
  * integer matrix products, scipy CSR products and numpy float64 matmul for special cases;
  * the average-bit values printed in the paper (tests/golden/paper_avg_bits.txt);
  * the round-trip bound of uniform quantization (Sec. 2.2 eqs. 2-5).
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import brute
import mpq_synth as synth
import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_avg_bits.txt")


def read_gold():
    out = {}
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, val, dec, params, _ = [s.strip() for s in line.split("|", 4)]
            out[key] = (float(val), int(dec), params)
    return out


# ---------------------------------------------------------------- conversions vs numpy's half

def test_half_to_float_all_patterns_match_numpy():
    allh = np.arange(65536, dtype=np.uint16)
    ref = allh.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(h)) for h in allh], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_float_to_half_matches_numpy_on_edges_and_random():
    rng = np.random.default_rng(1)
    bits = rng.integers(0, 2**32, size=200000, dtype=np.uint64).astype(np.uint32)
    # values around every half boundary: midpoints between consecutive halves and their neighbours
    h = np.arange(0, 0x7C00, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0
    mid = ((lo + hi) / 2).astype(np.float32)
    near = np.concatenate([mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9)),
                           -mid, np.float32([0.0, -0.0, 65504, 65519.99, 65520, 65536, 1e30, -1e30,
                                             2**-24, 2**-25, 2**-25 * 1.0001, 2**-26, 1e-45])])
    vals = np.concatenate([bits.view(np.float32), near.astype(np.float32)])
    vals = vals[~np.isnan(vals)]
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v)) for v in vals], dtype=np.uint16)
    bad = np.nonzero(got != ref)[0]
    assert bad.size == 0, (vals[bad[:5]], got[bad[:5]], ref[bad[:5]])


def test_round_binary_of_brute_agrees_with_numpy_half():
    # pins the brute-force rounding itself to an independent library before it is used as a pin
    rng = np.random.default_rng(2)
    vals = np.concatenate([rng.normal(0, 1, 2000), rng.normal(0, 1e-6, 2000), rng.normal(0, 3e4, 500)])
    for v in vals.astype(np.float64):
        fr = brute.round_binary(Fraction(float(v)), brute.F16)
        with np.errstate(over="ignore"):
            ref = int(np.float64(v).astype(np.float16).view(np.uint16))
        got = brute.fraction_to_half_bits(fr)
        if (ref & 0x7FFF) == 0:
            assert (got & 0x7FFF) == 0
        else:
            assert got == ref


# ---------------------------------------------------------------- per-element dequantization

def _np_scale(s_int, z2b, s2b):
    z2 = np.uint16(z2b).view(np.float16).astype(np.float32)
    s2 = np.uint16(s2b).view(np.float16).astype(np.float32)
    t = np.float32(np.float32(s_int) - z2)
    with np.errstate(over="ignore", invalid="ignore"):
        return int(np.float32(t * s2).astype(np.float16).view(np.uint16))


def test_scale_dequant_exhaustive_s_int_sampled_pairs():
    rng = np.random.default_rng(3)
    pairs = [(0x0000, 0x3C00), (0x8000, 0x3C00), (0x3800, 0x1400), (0x3BFF, 0x0001), (0x5BF8, 0x7BFF),
             (0x3C00, 0xBC00), (0x0001, 0x0400), (0x57F8, 0x03FF)]
    pairs += [(int(a), int(b)) for a, b in zip(synth.f16_bits(rng.random(40)),
                                               synth.f16_bits(np.exp(rng.normal(-6, 0.5, 40))))]
    pairs += [(int(a), int(b)) for a, b in rng.integers(0, 0x7C00, size=(40, 2))]
    for z2b, s2b in pairs:
        for s_int in range(256):
            got = oracle.scale_dequant(s_int, z2b, s2b)
            ref = _np_scale(s_int, z2b, s2b)
            assert got == ref, (s_int, hex(z2b), hex(s2b), hex(got), hex(ref))
            fr = brute.scale_dequant(s_int, z2b, s2b)
            if isinstance(fr, str):
                assert got == brute.fraction_to_half_bits(fr)
            elif fr == 0:
                assert (got & 0x7FFF) == 0
            else:
                assert got == brute.fraction_to_half_bits(fr)


def test_scale_identity_case():
    # z2 = 0, s2 = 1  ->  s1 = s_int exactly (all integers up to 255 are halves)
    for s_int in range(256):
        got = oracle.scale_dequant(s_int, 0x0000, 0x3C00)
        assert np.uint16(got).view(np.float16) == np.float16(s_int)


def test_scale_within_one_ulp_of_exact_real_value():
    # The op sequence (two fp32 ops then one half rounding) is a definition the paper leaves open;
    # whatever sequence is chosen must stay within one half ulp-step of the exactly rounded value.
    rng = np.random.default_rng(4)
    z2s = synth.f16_bits(rng.random(64))
    s2s = synth.f16_bits(np.exp(rng.normal(-6, 0.5, 64)))
    worst = 0
    for z2b, s2b in zip(z2s, s2s):
        for s_int in range(0, 256, 5):
            got = oracle.scale_dequant(s_int, int(z2b), int(s2b))
            exact = brute.round_binary((Fraction(s_int) - brute.half_bits_to_fraction(int(z2b)))
                                       * brute.half_bits_to_fraction(int(s2b)), brute.F16)
            if exact == 0:
                continue
            eb = brute.fraction_to_half_bits(exact)
            worst = max(worst, abs(int(got & 0x7FFF) - int(eb & 0x7FFF)))
            assert (got & 0x8000) == (eb & 0x8000)
    assert worst <= 1


def test_weight_dequant_all_codes_zeros_many_scales():
    rng = np.random.default_rng(5)
    s1s = list(rng.integers(0, 0x7C00, size=300)) + [0x0001, 0x03FF, 0x0400, 0x7BFF, 0x3555, 0x0000]
    s1s += [int(s) | 0x8000 for s in s1s[:100]]
    z1s = list(range(0, 16)) + [17, 63, 64, 127, 128, 200, 254, 255]
    for s1 in s1s:
        s1f = np.uint16(s1).view(np.float16).astype(np.float32)
        s1q = brute.half_bits_to_fraction(int(s1))
        for z1 in z1s:
            for code in range(16):
                got = oracle.weight_dequant(code, z1, int(s1))
                with np.errstate(over="ignore"):
                    ref = int(np.float32(np.float32(code - z1) * s1f).astype(np.float16).view(np.uint16))
                assert got == ref, (code, z1, hex(int(s1)), hex(got), hex(ref))
                fr = brute.round_binary(Fraction(code - z1) * s1q, brute.F16)
                if not isinstance(fr, str) and fr != 0:
                    assert got == brute.fraction_to_half_bits(fr)


def test_weight_product_is_a_single_rounding_native_half_multiply():
    # |d| <= 255 has <= 8 significant bits and a half 11, so the binary32 product is exact and the
    # result equals a native half multiply; numpy float16 multiplication is that operation.
    rng = np.random.default_rng(6)
    s1 = rng.integers(0, 0x7C00, size=5000).astype(np.uint16)
    d = rng.integers(-255, 16, size=5000)
    with np.errstate(over="ignore"):
        ref = (d.astype(np.float16) * s1.view(np.float16)).view(np.uint16)
    for i in range(5000):
        code, z1 = (int(d[i]), 0) if d[i] >= 0 else (0, int(-d[i]))
        assert oracle.weight_dequant(code, z1, int(s1[i])) == int(ref[i])


def test_outlier_add_matches_numpy_half_add():
    rng = np.random.default_rng(7)
    a = rng.integers(0, 0x7C00, size=4000).astype(np.uint16) | (rng.integers(0, 2, 4000).astype(np.uint16) << 15)
    b = synth.f16_bits(rng.normal(0, 0.5, 4000))
    with np.errstate(over="ignore"):
        ref = (a.view(np.float16) + b.view(np.float16)).view(np.uint16)
    for i in range(4000):
        assert oracle.add_outlier(int(a[i]), int(b[i])) == int(ref[i])


# ---------------------------------------------------------------- whole-matrix brute force

def _tiny(seed, N, K, g1, g2, f4, p_o, z1_full=False, is4=None):
    spec = synth.MatrixSpec("t", N, K, g1, g2, f4, p_o, seed)
    return synth.make_matrix(spec, z1_full_range=z1_full, is4=is4)


@pytest.mark.parametrize("N,K,g1,g2,g2_axis,f4,p_o,z1_full", [
    (5, 128, 16, 2, 0, 0.25, 0.05, False),
    (3, 192, 64, 16, 0, 0.34, 0.03, True),
    (7, 96, 16, 4, 0, 0.5, 0.1, True),     # G = 6, S = 2 with a short tail group
    (6, 64, 16, 1, 0, 0.0, 0.0, False),
    (4, 256, 64, 2, 0, 1.0, 0.0, False),
    (7, 64, 16, 3, 1, 0.25, 0.05, True),   # second-order groups along the rows, short tail
    (8, 128, 32, 4, 1, 0.25, 0.02, False),
])
def test_matrix_against_rational_brute_force(N, K, g1, g2, g2_axis, f4, p_o, z1_full):
    lg = _tiny(100 + N + K + g2, N, K, g1, g2, f4, p_o, z1_full)
    G = K // g1
    if g2_axis == 1:  # second-order arrays have shape [ceil(N/g2), G] for this axis
        rng = np.random.default_rng(9)
        R = -(-N // g2)
        lg.s2 = synth.f16_bits(np.exp(rng.normal(-6, 0.5, size=(R, G))))
        lg.z2 = synth.f16_bits(rng.random(size=(R, G)))
    m = oracle.Matrix.from_logical(lg, g2_axis)
    assert m.validate() == 0
    Wd = m.dequant(False)
    Wf = m.dequant(True)
    WB = brute.dequant(N, K, g1, g2, g2_axis, lg.codes, lg.s_int, lg.z1, lg.s2, lg.z2)
    for n in range(N):
        for k in range(K):
            fr = WB[n][k]
            if fr == 0:
                assert (int(Wd[n, k]) & 0x7FFF) == 0
            else:
                assert int(Wd[n, k]) == brute.fraction_to_half_bits(fr), (n, k)
    # outliers: additive, only at CSR positions
    diff = np.nonzero(Wf != Wd)
    at = set()
    for n in range(N):
        for e in range(lg.row_ptr[n], lg.row_ptr[n + 1]):
            c = int(lg.col[e])
            at.add((n, c))
            want = brute.round_binary(WB[n][c] + brute.half_bits_to_fraction(int(lg.val[e])), brute.F16)
            if want != 0:
                assert int(Wf[n, c]) == brute.fraction_to_half_bits(want)
    assert set(zip(diff[0].tolist(), diff[1].tolist())) <= at
    # product, exact rationals vs binary64 accumulation
    X = synth.make_x(5, 2, K)
    Y = m.gemm(X)
    YB = brute.gemm(WB, lg.row_ptr, lg.col, lg.val, X)
    for mm in range(2):
        for n in range(N):
            ref = float(YB[mm][n])
            scale = float(sum(abs(WB[n][k] * brute.half_bits_to_fraction(int(X[mm][k]))) for k in range(K))) + 1e-30
            assert abs(Y[mm, n] - ref) <= 1e-13 * scale, (mm, n, Y[mm, n], ref)


def test_every_is4_subset_for_four_groups():
    N, K, g1, g2 = 2, 64, 16, 2
    for mask in range(16):
        is4 = np.array([(mask >> g) & 1 for g in range(4)], dtype=np.uint8)
        lg = _tiny(200 + mask, N, K, g1, g2, 0.0, 0.08, True, is4=is4)
        m = oracle.Matrix.from_logical(lg)
        assert m.validate() == 0
        # outliers only in 2-bit groups
        assert not np.any(is4[lg.col // g1])
        Wd = m.dequant(False)
        WB = brute.dequant(N, K, g1, g2, 0, lg.codes, lg.s_int, lg.z1, lg.s2, lg.z2)
        for n in range(N):
            for k in range(K):
                if WB[n][k] != 0:
                    assert int(Wd[n, k]) == brute.fraction_to_half_bits(WB[n][k])


# ---------------------------------------------------------------- special cases with library answers

def test_identity_scales_reduce_to_integer_matmul():
    N, K, g1, g2 = 24, 256, 64, 2
    lg = _tiny(11, N, K, g1, g2, 0.25, 0.0)
    lg.s_int[:] = 1
    lg.z1[:] = 0
    lg.s2[:] = 0x3C00
    lg.z2[:] = 0
    m = oracle.Matrix.from_logical(lg)
    Wd = m.dequant(False).view(np.float16)
    assert np.array_equal(Wd.astype(np.int64), lg.codes.astype(np.int64))
    rng = np.random.default_rng(12)
    xi = rng.integers(-3, 4, size=(3, K))
    X = xi.astype(np.float16).view(np.uint16)
    Y = m.gemm(X)
    assert np.array_equal(Y, (xi @ lg.codes.astype(np.int64).T).astype(np.float64))


def test_codes_equal_zero_point_reduces_to_csr_product():
    N, K, g1, g2 = 40, 512, 64, 4
    lg = _tiny(13, N, K, g1, g2, 0.25, 0.03)
    lg.z1[:] = np.minimum(lg.z1, 3)
    lg.codes[:] = np.repeat(lg.z1, g1, axis=1)
    m = oracle.Matrix.from_logical(lg)
    assert m.validate() == 0
    X = synth.make_x(14, 2, K)
    Y = m.gemm(X)
    A = sp.csr_matrix((lg.val.view(np.float16).astype(np.float64), lg.col.astype(np.int64),
                       lg.row_ptr.astype(np.int64)), shape=(N, K))
    ref = (A @ X.view(np.float16).astype(np.float64).T).T
    assert lg.nnz > 0
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


def test_gemm_equals_numpy_matmul_of_dequantized_matrix():
    lg = _tiny(15, 64, 1024, 64, 16, 0.125, 0.005)
    m = oracle.Matrix.from_logical(lg)
    X = synth.make_x(16, 3, 1024)
    Y = m.gemm(X)
    Wd = m.dequant(False).view(np.float16).astype(np.float64)
    Xf = X.view(np.float16).astype(np.float64)
    A = sp.csr_matrix((lg.val.view(np.float16).astype(np.float64), lg.col.astype(np.int64),
                       lg.row_ptr.astype(np.int64)), shape=(64, 1024))
    ref = Xf @ Wd.T + (A @ Xf.T).T
    np.testing.assert_allclose(Y, ref, rtol=1e-11, atol=1e-9)
    # threads do not change the result, rows restrict it
    Y2 = m.gemm(X, threads=4)
    assert np.array_equal(Y, Y2)
    Y3 = m.gemm(X, rows=(10, 20))
    assert np.array_equal(Y3[:, 10:20], Y[:, 10:20]) and not Y3[:, :10].any() and not Y3[:, 20:].any()


def test_pure_2bit_and_pure_4bit_are_plain_groupwise_quantization():
    # with f4 = 0 or 1 the format is ordinary group-wise uniform quantization: W = (c - z) * s per group
    for f4, hi in ((0.0, 3), (1.0, 15)):
        lg = _tiny(17, 16, 256, 64, 16, f4, 0.0)
        assert lg.codes.max() <= hi
        m = oracle.Matrix.from_logical(lg)
        s1 = m.scales().view(np.float16).astype(np.float64)
        ref = (lg.codes.astype(np.float64) - np.repeat(lg.z1, 64, axis=1)) * np.repeat(s1, 64, axis=1)
        got = m.dequant(False).view(np.float16).astype(np.float64)
        # each weight is the half nearest to (c - z) * s1
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0**-11 + 2.0**-25)


def test_uniform_quantization_round_trip_bound():
    # Sec. 2.2 eqs. 2-4 quantize, eq. 5 (the oracle) dequantizes: |w - w_hat| <= s/2 for unclamped values
    rng = np.random.default_rng(18)
    N, K, g1 = 8, 256, 64
    G = K // g1
    for nbits in (2, 4):
        w = rng.normal(0, 0.02, size=(N, K))
        wg = w.reshape(N, G, g1)
        wmax, wmin = wg.max(axis=2), wg.min(axis=2)
        s = ((wmax - wmin) / (2**nbits - 1)).astype(np.float16)         # "scaling factor is half"
        sf = s.astype(np.float64)
        z = np.rint(-wmin / sf)
        q = np.clip(np.rint(wg / sf[..., None]) + z[..., None], 0, 2**nbits - 1)
        unclamped = (np.rint(wg / sf[..., None]) + z[..., None] == q)
        # express s through the second-order pair exactly: s_int = 1, z2 = 0, s2 = s
        m = oracle.Matrix(N, K, g1, 1, np.full(G, nbits == 4, np.uint8), q.reshape(N, K).astype(np.uint8),
                          np.ones((N, G), np.uint8), z.astype(np.uint8), s.view(np.uint16),
                          np.zeros((N, G), np.uint16), np.zeros(N + 1, np.int32), np.zeros(0, np.uint16),
                          np.zeros(0, np.uint16))
        assert m.validate() == 0
        what = m.dequant(False).view(np.float16).astype(np.float64).reshape(N, G, g1)
        err = np.abs(what - wg)
        bound = sf[..., None] / 2 * (1 + 2e-3) + 1e-6
        assert np.all(err[unclamped] <= np.broadcast_to(bound, err.shape)[unclamped])


def test_validate_rejects_malformed_inputs():
    lg = _tiny(19, 8, 256, 64, 2, 0.25, 0.05)
    m = oracle.Matrix.from_logical(lg)
    assert m.validate() == 0
    g4 = int(np.nonzero(lg.is4)[0][0])
    g2b = int(np.nonzero(lg.is4 == 0)[0][0])
    bad = oracle.Matrix.from_logical(lg)
    bad.codes[0, g2b * 64] = 4
    assert bad.validate() == 2
    bad = oracle.Matrix.from_logical(lg)
    r = int(np.nonzero(np.diff(lg.row_ptr) > 0)[0][0])
    bad.col[lg.row_ptr[r]] = g4 * 64
    assert bad.validate() in (3, 4)
    bad = oracle.Matrix.from_logical(lg)
    bad.row_ptr[1] = bad.row_ptr[-1] + 5
    assert bad.validate() == 3


# ---------------------------------------------------------------- average bits printed in the paper

def test_average_bits_printed_in_the_paper():
    g = read_gold()
    v, dec, _ = g["mixed_25pct"]
    assert round(oracle.avg_bits_mixed(0.75, 4, 16, 16), dec) == v
    assert abs(oracle.avg_bits_mixed(0.75, 4, 16, 16) - 2.83984375) < 1e-12
    v, dec, _ = g["mixed_10pct"]
    assert abs(oracle.avg_bits_mixed(0.90, 4, 16, 16) - v) < 0.01      # 2.6078 printed as 2.60
    v, dec, _ = g["ablation_25"]
    assert abs(oracle.avg_bits_mixed(0.75, 4, 16, 16) - v) < 0.011
    for key, ratio in (("outlier_1p5", 0.015), ("outlier_0p2", 0.002), ("outlier_0p5", 0.005)):
        v, dec, _ = g[key]
        assert round(oracle.outlier_bits(ratio), dec) == v
    v, dec, _ = g["with_outliers"]
    tot = oracle.avg_bits_mixed(0.75, 4, 16, 16) + oracle.outlier_bits(0.002)
    assert tot <= v <= tot + 0.02 + 0.005
    # first- and second-order formulas of Sec. 2.2, by hand: 2 + 18/16 and 2 + 6/16 + 20/256
    assert oracle.avg_bits_first_order(2, 16) == 3.125
    assert oracle.avg_bits_second_order(2, 4, 16, 16) == 2 + 6 / 16 + 20 / 256
    assert g["align_unit"][0] == 3 * 16 * 2 + 8 * 4 and g["align_second"][0] == 8 * 4
    assert g["align_meta"][0] == 3 * 2 + 4 + 3 + 3


def test_stored_bits_match_byte_count_of_the_arrays():
    for cfg in (0, 1, 3):
        for spec in synth.config_specs(cfg):
            nnz = int(round(spec.p_o * spec.N * (spec.G - spec.n4) * spec.g1))
            by = synth.stored_bytes(spec, spec.n4, nnz)
            want = 8.0 * by["total"] / (spec.N * spec.K)
            got = oracle.avg_bits_stored(spec.N, spec.K, spec.g1, spec.g2, spec.n4, nnz)
            assert abs(got - want) < 1e-9
    # the headline layer moves about 2.62 bits per weight
    specs = synth.config_specs(1)
    tot = sum(synth.stored_bytes(s, s.n4, int(round(s.p_o * s.N * (s.G - s.n4) * s.g1)))["total"] for s in specs)
    assert abs(8.0 * tot / sum(s.N * s.K for s in specs) - 2.62) < 0.01
