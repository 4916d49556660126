"""The paper's aligned metadata packing (Sec. 3.3 "Memory Alignment": one 16-bit word for the zero points and
scales of three 2-bit groups, two of the scales clipped to 3 bits; a byte-padded Ns-bit second-order zero):
the oracle's reading of it pinned by brute force and by the paper's bit counts, and the library's packer held
to the same rules (CPU only)."""
import numpy as np
import pytest

import mpq_synth as synth
import oracle
import paper_2311_16442_amd as mpq


def clip_brute(is4, s_int):
    """Plain loops: count a row's 2-bit groups in K order; the 2nd and 3rd of every three saturate at 7, every
    other scale code at 15."""
    out = np.array(s_int, dtype=np.uint8)
    for n in range(out.shape[0]):
        seen = 0
        for g in range(out.shape[1]):
            lim = 15
            if not is4[g]:
                lim = 15 if seen % 3 == 0 else 7
                seen += 1
            out[n, g] = min(int(out[n, g]), lim)
    return out


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_scale_clipping_matches_brute_force_and_is_idempotent(seed):
    rng = np.random.default_rng(seed)
    N, G = 7, 23
    is4 = (rng.random(G) < 0.3).astype(np.uint8)
    s = rng.integers(0, 256, size=(N, G), dtype=np.uint8)
    got = oracle.clip_scales(N, G * 16, 16, is4, s)
    assert np.array_equal(got, clip_brute(is4, s))
    assert np.array_equal(oracle.clip_scales(N, G * 16, 16, is4, got), got)
    two = np.nonzero(is4 == 0)[0]
    assert got[:, two[0::3]].max() <= 15 and (two.size < 2 or got[:, two[1::3]].max() <= 7) and (two.size < 3 or got[:, two[2::3]].max() <= 7)
    assert got[:, is4 != 0].max(initial=0) <= 15
    # values that already fit are left alone
    small = rng.integers(0, 8, size=(N, G), dtype=np.uint8)
    assert np.array_equal(oracle.clip_scales(N, G * 16, 16, is4, small), small)


def test_the_word_has_sixteen_bits():
    # three 2-bit zero points, one 4-bit and two 3-bit scales (Sec. 3.3, Scale Clipping)
    assert 3 * 2 + 4 + 3 + 3 == 16


@pytest.mark.parametrize("axis", [0, 1])
def test_validation_of_oracle_and_packer_agree(axis):
    spec = synth.MatrixSpec("a", 40, 512, 16, 16, 0.25, 0.01, 99, axis, 1)
    lg = synth.make_matrix(spec)
    assert oracle.validate_aligned(40, 512, 16, 16, lg.is4, lg.s_int, lg.z1, lg.z2, axis) == 0
    mpq.pack_logical(lg)                                   # accepted
    g2bit = np.nonzero(lg.is4 == 0)[0]

    def refused(**change):
        arrs = dict(s_int=lg.s_int.copy(), z1=lg.z1.copy(), z2=lg.z2.copy())
        for k, (idx, v) in change.items():
            arrs[k][idx] = v
        assert oracle.validate_aligned(40, 512, 16, 16, lg.is4, arrs["s_int"], arrs["z1"], arrs["z2"], axis) == 5
        with pytest.raises(mpq.MpqError) as e:
            mpq.pack(40, 512, 16, 16, lg.is4, lg.codes, arrs["s_int"], arrs["z1"], lg.s2, arrs["z2"], lg.row_ptr, lg.col, lg.val,
                     axis, mpq.META_PAPER)
        assert e.value.status == mpq.MPQ_ERR_CODE_RANGE

    refused(z1=((3, g2bit[0]), 4))                        # a 2-bit zero point of 4
    refused(s_int=((5, g2bit[1]), 8))                     # second group of a triple: 3 bits
    refused(s_int=((5, g2bit[2]), 8))                     # third group of a triple: 3 bits
    refused(s_int=((5, g2bit[3]), 16))                    # first group of the next triple: 4 bits
    refused(z2=((0, 0), synth.f16_bits(np.array([2.5]))[0]))    # not an integer
    refused(z2=((0, 0), synth.f16_bits(np.array([16.0]))[0]))   # beyond Ns = 4 bits
    ok = lg.s_int.copy()
    ok[5, g2bit[3]] = 15                                   # the first of a triple may use all 4 bits
    assert oracle.validate_aligned(40, 512, 16, 16, lg.is4, ok, lg.z1, lg.z2, axis) == 0
    # group sizes other than the paper's 16 are not part of this packing
    lg64 = synth.make_matrix(synth.MatrixSpec("b", 16, 512, 64, 16, 0.25, 0.0, 98))
    with pytest.raises(mpq.MpqError) as e:
        mpq.pack(16, 512, 64, 16, lg64.is4, lg64.codes, lg64.s_int % 8, lg64.z1 % 4, lg64.s2, synth.f16_bits(np.ones(lg64.z2.shape)),
                 lg64.row_ptr, lg64.col, lg64.val, 0, mpq.META_PAPER)
    assert e.value.status == mpq.MPQ_ERR_UNSUPPORTED


def test_stored_bits_of_the_aligned_format_against_the_papers_count():
    # the paper's operating point: g1 = g2 = 16 with pairs shared by 16 rows, a quarter of the groups 4-bit
    N, K, g1, g2 = 4096, 4096, 16, 16
    G = K // g1
    n4 = G // 4
    stored = oracle.avg_bits_stored_aligned(N, K, g1, g2, n4, 0, g2_axis=1)
    assert abs(stored - mpq.avg_bits(N, K, g1, g2, n4, 0, mode=0, g2_axis=1, meta=mpq.META_PAPER)) < 1e-12
    # by hand: codes, 16 bits per three 2-bit groups, 8 bits per 4-bit group, 24 bits per pair, row pointers
    n2 = G - n4
    by_hand = (N * g1 * (2 * n2 + 4 * n4) + N * (16 * ((n2 + 2) // 3) + 8 * n4) + 24 * (N // g2) * G + 32 * (N + 1)) / (N * K)
    assert abs(stored - by_hand) < 1e-12
    # the 2-bit groups' share against the paper's formula (Sec. 3.3: alignment costs less than 0.02 bits):
    # 2 + 16 / 48 + 24 / 256 per weight of a 2-bit group against 2 + (2 + 4) / 16 + (4 + 16) / 256
    alpha = n2 / G
    ours_2bit = alpha * (2 + 16 / (3 * g1) + 24 / (g1 * g2))
    paper_2bit = alpha * oracle.avg_bits_second_order(2, 4, g1, g2)
    assert abs(ours_2bit - paper_2bit) < 0.02
    # what is left is what the paper's formula leaves out: the scale, zero point and second-order pair of the
    # 4-bit groups (8 / 16 + 24 / 256 per weight of a 4-bit group) and the row pointers
    rest = stored - ours_2bit - (1 - alpha) * 4
    assert abs(rest - ((1 - alpha) * (8 / g1 + 24 / (g1 * g2)) + 32 * (N + 1) / (N * K))) < 1e-9
    # so the format stores 2.97 bits per weight where the byte-wide metadata stores 3.63
    assert 2.96 < stored < 2.98 and 3.6 < oracle.avg_bits_stored(N, K, g1, g2, n4, 0, g2_axis=1) < 3.7


def test_decoding_the_aligned_format_is_the_same_formula():
    # the logical arrays of a matrix in the aligned format are plain logical arrays: the oracle decodes
    # them with the definition, whatever the storage
    spec = synth.MatrixSpec("c", 24, 320, 16, 16, 0.2, 0.02, 97, 1, 1)
    lg = synth.make_matrix(spec)
    om = oracle.Matrix.from_logical(lg)
    W = om.dequant(False).view(np.float16).astype(np.float64)
    s1 = om.scales().view(np.float16).astype(np.float64).reshape(24, 20)
    d = lg.codes.astype(np.int64) - np.repeat(lg.z1.astype(np.int64), 16, axis=1)
    assert np.allclose(W, d * np.repeat(s1, 16, axis=1), rtol=2 ** -10, atol=0)
