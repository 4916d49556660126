"""The reference quantizer (Sec. 2.2 eqs. 2-5, Sec. 3.3, Sec. 4.3): pins of the oracle's version
against what the equations fix, and the library's host quantizer against the oracle bit for bit."""
import numpy as np
import pytest

import oracle
import paper_2311_16442_amd as mpq
from oracle import quantizer as oq


def heavy_tailed(N, K, seed, hot_groups=(), g1=64):
    rng = np.random.default_rng(seed)
    W = (rng.standard_t(df=5, size=(N, K)) * 0.02).astype(np.float32)
    for g in hot_groups:
        W[:, g * g1:(g + 1) * g1] *= 6.0
    return W


def dequantize(q, N, K, g1, g2, axis):
    om = oracle.Matrix(N, K, g1, g2, q["is4"], q["codes"], q["s_int"], q["z1"], q["s2"], q["z2"],
                       q["row_ptr"], q["col"], q["val"], g2_axis=axis)
    assert om.validate() == 0
    half = lambda a: a.view(np.float16).astype(np.float64)
    return half(om.dequant(False)), half(om.dequant(True)), half(om.scales())


def test_uniform_quantization_round_trip_bound():
    # eqs. 2-5: a weight whose code is not clamped is reproduced to within half a step
    N, K, g1, g2 = 24, 512, 64, 4
    W = heavy_tailed(N, K, 1)
    q = oq.quantize(W, g1, g2, 0, 0.0)
    Wd, _, s1 = dequantize(q, N, K, g1, g2, 0)
    assert not q["is4"].any() and q["codes"].max() <= 3 and q["row_ptr"][-1] == 0
    step = np.repeat(s1, g1, axis=1)
    z = np.repeat(q["z1"].astype(np.float64), g1, axis=1)
    unclamped = np.rint(W.astype(np.float64) / step) + z
    inside = (unclamped >= 0) & (unclamped <= 3)
    assert inside.mean() > 0.9                     # the 8-bit scale rarely shrinks the range
    err = np.abs(W - Wd)
    assert np.all(err[inside] <= 0.5 * step[inside] * (1 + 1e-9) + np.abs(Wd[inside]) * 2.0 ** -11)
    # eq. 3: the zero point is an N-bit integer; eq. 2: the step spans the range of the group
    assert q["z1"].max() <= 3
    rng_g = W.reshape(N, K // g1, g1).max(axis=2) - W.reshape(N, K // g1, g1).min(axis=2)
    assert np.all(np.abs(3 * s1 - rng_g) <= rng_g * (2 / 255 + 2.0 ** -10) + 1e-12)


def test_sensitive_groups_become_four_bit_and_reduce_the_error():
    N, K, g1, g2 = 32, 1024, 64, 16
    hot = (3, 7, 12)
    W = heavy_tailed(N, K, 2, hot_groups=hot)
    q = oq.quantize(W, g1, g2, 3, 0.0)
    assert sorted(np.nonzero(q["is4"])[0]) == list(hot)            # eq. 9: largest sum of squares
    for g in range(K // g1):
        assert q["codes"][:, g * g1:(g + 1) * g1].max() <= (15 if q["is4"][g] else 3)
    rel = lambda n4: np.linalg.norm(W - dequantize(oq.quantize(W, g1, g2, n4, 0.0), N, K, g1, g2, 0)[0]) / np.linalg.norm(W)
    e0, e3, e8 = rel(0), rel(3), rel(8)
    assert e8 < e3 < e0                                             # Sec. 3.3: 4-bit groups where the range is large


def test_outliers_stay_in_two_bit_groups_and_restore_the_weight():
    N, K, g1, g2 = 16, 512, 64, 8
    W = heavy_tailed(N, K, 3, hot_groups=(1,))
    planted = [(0, 200), (0, 300), (5, 10), (9, 500)]
    for n, k in planted:
        W[n, k] = 3.0
    W[4, 70] = 9.0                                                  # inside the (future) 4-bit group 1
    p_o = 2 / (K - g1)                                              # two outliers per row
    q = oq.quantize(W, g1, g2, 1, p_o)
    assert list(np.nonzero(q["is4"])[0]) == [1]
    rp, col = q["row_ptr"], q["col"]
    assert np.all(np.diff(rp) == 2)
    assert not np.any(q["is4"][col // g1])                          # Sec. 4.3: only 2-bit groups
    assert {200, 300} == set(col[rp[0]:rp[1]]) and 10 in col[rp[5]:rp[6]] and 500 in col[rp[9]:rp[10]]
    Wd, Wfull, _ = dequantize(q, N, K, g1, g2, 0)
    for n in range(N):
        for e in range(rp[n], rp[n + 1]):
            k = int(col[e])
            assert abs(Wfull[n, k] - W[n, k]) <= abs(W[n, k]) * 2.0 ** -10 + 1e-6   # dense + sparse = the weight
            assert np.all(np.diff(col[rp[n]:rp[n + 1]].astype(int)) > 0)
    # the outliers do not widen their group's range: the rest of the group is quantized finely
    assert np.abs(W[0, 192:256] - Wd[0, 192:256])[np.arange(64) != 8].max() < 0.05
    e_with = np.linalg.norm((W - Wfull)[:, q["is4"].repeat(g1) == 0])
    q0 = oq.quantize(W, g1, g2, 1, 0.0)
    e_without = np.linalg.norm((W - dequantize(q0, N, K, g1, g2, 0)[0])[:, q0["is4"].repeat(g1) == 0])
    assert e_with < 0.95 * e_without


CASES = [
    # N, K, g1, g2, n4, p_o, axis
    (24, 512, 64, 4, 2, 0.01, 0),
    (37, 704, 64, 16, 3, 0.005, 0),
    (40, 512, 16, 16, 8, 0.01, 1),
    (33, 480, 32, 4, 3, 0.02, 1),
    (16, 256, 128, 2, 1, 0.0, 0),
    (16, 256, 64, 1, 0, 0.05, 0),       # every scale is its own second-order group
]


@pytest.mark.parametrize("N,K,g1,g2,n4,p_o,axis", CASES)
def test_library_quantizer_matches_oracle_bit_for_bit(N, K, g1, g2, n4, p_o, axis):
    W = heavy_tailed(N, K, 10 + N + K, hot_groups=(1,), g1=g1)
    W[0, :g1] = 0.25                                                # a constant group
    W[1, :g1] = 0.0                                                 # an all-zero group
    ref = oq.quantize(W, g1, g2, n4, p_o, axis)
    got = mpq.quantize(W, g1, g2, n4, p_o, axis)
    for name in ("is4", "codes", "s_int", "z1", "s2", "z2", "row_ptr", "col", "val"):
        assert np.array_equal(got[name], ref[name]), name
    # and what it produces packs
    pk = mpq.pack(N, K, g1, g2, g2_axis=axis, **got)
    assert pk.nnz == int(ref["row_ptr"][-1]) and pk.n4 == n4


def test_quantizer_rejects_bad_arguments():
    W = np.zeros((16, 256), np.float32)
    for kw in (dict(g1=48), dict(n4=5), dict(p_o=-0.1), dict(p_o=1.5)):
        args = dict(g1=64, g2=4, n4=1, p_o=0.0)
        args.update(kw)
        with pytest.raises(mpq.MpqError):
            mpq.quantize(W, **args)
