"""CPU oracle of the reference quantizer (test infrastructure, not product code).

Plain numpy in binary64, in the paper's notation: uniform quantization of a group (Sec. 2.2,
eqs. 2-5), second-order quantization of the scales (Sec. 2.2 / 3.3), 4-bit groups chosen by the
sensitivity of the input-channel groups (Sec. 3.3, eq. 9, with the Hessian term set to one: no
calibration data), outliers kept only inside 2-bit groups (Sec. 4.3).  Only tests import this.

Where the paper is silent the readings are (the library's quantizer documents the same list):
  - sensitivity of group g: S_g = sum over all rows and the group's columns of w^2; the n4 groups
    with the largest S_g are 4-bit, ties to the lower index;
  - outliers: per row the round(p_o * #2-bit columns) weights of largest |w| among the row's 2-bit
    columns, ties to the lower column; they do not take part in the group's min / max;
  - eq. 2-3 with the range over the non-outlier weights; a constant group uses s = |w| (1 if 0);
    the zero point is clamped to [0, 2^N - 1] (it is an N-bit integer);
  - scales are quantized to 8 bits (the format's uint8): s2 = fp16(max((s_max - s_min) / 255,
    s_max / 2047)), z2 = fp16(round(-s_min / s2)), s_int = clamp(round(s / s2) + z2); the second
    term keeps |z2| <= 2047, an integer that fp16 holds exactly, when the scales of a group are
    nearly equal;
  - zero points and codes are computed against the scale as the decoder will reconstruct it
    (s1 = fp16((s_int - z2) * s2)), so that quantize -> dequantize is consistent;
  - an outlier's stored value is fp16(w - dequantized dense value): dense + sparse (Sec. 2.3).
round() is round-half-to-even throughout.
"""
from __future__ import annotations

import numpy as np

import oracle


def _half(a):
    """fp16 bit patterns of binary64 values (round to nearest even, through binary32 like the decoder)."""
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float16).view(np.uint16)


def _half_value(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def quantize(W, g1, g2, n4, p_o, g2_axis=0):
    """Returns dict(is4, codes, s_int, z1, s2, z2, row_ptr, col, val) in the logical format."""
    W = np.asarray(W, dtype=np.float32).astype(np.float64)
    N, K = W.shape
    G = K // g1
    Wg = W.reshape(N, G, g1)
    # --- eq. 9 with a unit Hessian: sensitivity per input-channel group, largest n4 become 4-bit
    S = np.array([float(np.sum(Wg[:, g, :].astype(np.float64) ** 2)) for g in range(G)])
    order = sorted(range(G), key=lambda g: (-S[g], g))
    is4 = np.zeros(G, dtype=np.uint8)
    is4[order[:n4]] = 1
    bits = np.where(is4 != 0, 4, 2)
    # --- Sec. 4.3: outliers only inside 2-bit groups, largest magnitudes of each row
    cols2 = np.nonzero(np.repeat(is4, g1) == 0)[0]
    cnt = int(np.floor(p_o * cols2.size + 0.5))
    out_mask = np.zeros((N, K), dtype=bool)
    if cnt > 0:
        for n in range(N):
            mag = np.abs(W[n, cols2])
            pick = sorted(range(cols2.size), key=lambda q: (-mag[q], q))[:cnt]
            out_mask[n, cols2[pick]] = True
    # --- eq. 2: scale of every (row, group) from the range of its non-outlier weights
    keep = ~out_mask.reshape(N, G, g1)
    lo = np.where(keep, Wg, np.inf).min(axis=2)
    hi = np.where(keep, Wg, -np.inf).max(axis=2)
    empty = ~keep.any(axis=2)
    lo[empty] = 0.0
    hi[empty] = 0.0
    levels = (2.0 ** bits - 1.0)[None, :]
    s = (hi - lo) / levels
    const = s == 0.0
    s[const] = np.where(lo[const] != 0.0, np.abs(lo[const]), 1.0)
    # --- second-order quantization of the scales (8 bits) along the chosen axis
    if g2_axis == 0:
        S2 = -(-G // g2)
        blocks = [(slice(None), slice(j * g2, min((j + 1) * g2, G))) for j in range(S2)]
        shape2 = (N, S2)
    else:
        NB = -(-N // g2)
        blocks = [(slice(b * g2, min((b + 1) * g2, N)), slice(None)) for b in range(NB)]
        shape2 = (NB, G)
    s2 = np.zeros(shape2, dtype=np.uint16)
    z2 = np.zeros(shape2, dtype=np.uint16)
    s_int = np.zeros((N, G), dtype=np.uint8)
    for idx, (rs, gs) in enumerate(blocks):
        blk = s[rs, gs]
        axis = 1 if g2_axis == 0 else 0
        smin, smax = blk.min(axis=axis), blk.max(axis=axis)
        s2b = _half(np.maximum((smax - smin) / 255.0, smax / 2047.0))
        s2f = _half_value(s2b)
        s2f_safe = np.where(s2f == 0.0, 1.0, s2f)
        z2b = _half(np.rint(-smin / s2f_safe))
        z2f = _half_value(z2b)
        if g2_axis == 0:
            q = np.rint(blk / s2f_safe[:, None]) + z2f[:, None]
            s2[:, idx], z2[:, idx] = s2b, z2b
        else:
            q = np.rint(blk / s2f_safe[None, :]) + z2f[None, :]
            s2[idx, :], z2[idx, :] = s2b, z2b
        s_int[rs, gs] = np.clip(q, 0, 255).astype(np.uint8)
    # --- the scale as the decoder reconstructs it, then eq. 3-4 against that scale
    if g2_axis == 0:
        s2e, z2e = np.repeat(s2, g2, axis=1)[:, :G], np.repeat(z2, g2, axis=1)[:, :G]
    else:
        s2e, z2e = np.repeat(s2, g2, axis=0)[:N], np.repeat(z2, g2, axis=0)[:N]
    s1 = np.array([[oracle.scale_dequant(int(s_int[n, g]), int(z2e[n, g]), int(s2e[n, g])) for g in range(G)]
                   for n in range(N)], dtype=np.uint16)
    s1f = _half_value(s1)
    ok = s1f != 0.0
    s1_safe = np.where(ok, s1f, 1.0)
    z1 = np.where(ok, np.clip(np.rint(-lo / s1_safe), 0, levels), 0.0)
    codes = np.clip(np.rint(Wg / s1_safe[:, :, None]) + z1[:, :, None], 0, levels[:, :, None])
    codes = np.where(ok[:, :, None], codes, 0.0).astype(np.uint8).reshape(N, K)
    z1 = z1.astype(np.uint8)
    # --- outliers: the part of the weight the dense code does not carry (dense + sparse)
    row_ptr = np.zeros(N + 1, dtype=np.int32)
    col, val = [], []
    for n in range(N):
        ks = np.nonzero(out_mask[n])[0]
        row_ptr[n + 1] = row_ptr[n] + ks.size
        for k in ks:
            g = k // g1
            wd = _half_value(oracle.weight_dequant(int(codes[n, k]), int(z1[n, g]), int(s1[n, g])))
            col.append(k)
            val.append(int(_half(W[n, k] - float(wd))))
    return dict(is4=is4, codes=codes, s_int=s_int, z1=z1, s2=s2, z2=z2, row_ptr=row_ptr,
                col=np.array(col, dtype=np.uint16), val=np.array(val, dtype=np.uint16))
