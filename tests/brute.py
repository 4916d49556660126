"""Exact-rational brute force of the weight format, for tiny matrices only.

Independent of oracle/ and of the HIP library: every value is a fractions.Fraction, every
rounding goes through `round_binary`, a from-first-principles IEEE 754 round-to-nearest-even
for an arbitrary (precision, emin, emax) format, and all indexing is spelled out with Python
loops straight from the definitions (Sec. 2.2 eq. 5, Sec. 3.3, Algorithm 1, Sec. 2.3).
"""
from fractions import Fraction

F16 = (11, -14, 15)      # precision (bits incl. hidden), emin, emax
F32 = (24, -126, 127)


def half_bits_to_fraction(h: int) -> Fraction:
    sign = -1 if (h >> 15) & 1 else 1
    e = (h >> 10) & 0x1F
    m = h & 0x3FF
    if e == 0x1F:
        raise ValueError("inf/nan has no rational value")
    if e == 0:
        return sign * Fraction(m, 1 << 24)
    return sign * Fraction(1024 + m, 1024) * (Fraction(2) ** (e - 15))


def round_binary(v: Fraction, fmt):
    """Round v to the nearest value of a binary format, ties to even. Returns a Fraction, or
    +-'inf' (as a string) on overflow."""
    p, emin, emax = fmt
    if v == 0:
        return Fraction(0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e_eff = max(e, emin)
    quantum = Fraction(2) ** (e_eff - (p - 1))
    q = a / quantum
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    r = fl * quantum
    if r >= Fraction(2) ** (emax + 1):
        return "inf" if sign > 0 else "-inf"
    return sign * r


def fraction_to_half_bits(v) -> int:
    """Bit pattern of an exactly representable half (or +-inf)."""
    if v == "inf":
        return 0x7C00
    if v == "-inf":
        return 0xFC00
    if v == 0:
        return 0
    sign = 0x8000 if v < 0 else 0
    a = abs(v)
    if a < Fraction(1, 1 << 14):
        m = a * (1 << 24)
        assert m.denominator == 1
        return sign | int(m)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    m = a / (Fraction(2) ** e) * 1024 - 1024
    assert m.denominator == 1 and 0 <= m < 1024
    return sign | ((e + 15) << 10) | int(m)


def scale_dequant(s_int: int, z2_bits: int, s2_bits: int, signed_zero_from=None):
    """Second-order dequantization with the stated op sequence: fp32 subtract, fp32 multiply, half round.
    Returns (half bits or None when the result is a zero whose sign this model does not track, value)."""
    t = round_binary(Fraction(s_int) - half_bits_to_fraction(z2_bits), F32)
    u = round_binary(t * half_bits_to_fraction(s2_bits), F32)
    s1 = round_binary(u, F16)
    return s1


def weight_dequant(code: int, z1: int, s1):
    if isinstance(s1, str):
        d = code - z1
        if d == 0:
            return "nan"
        return s1 if d > 0 else ("-inf" if s1 == "inf" else "inf")
    return round_binary(Fraction(code - z1) * s1, F16)


def second_order_pair(n, g, g2, g2_axis):
    """(row, column) of the pair of (row n, K-group g) in the 2-D arrays s2 / z2: [N][S] when a pair covers
    g2 groups along K, [ceil(N / g2)][G] when it covers the same K-group of g2 rows."""
    return (n, g // g2) if g2_axis == 0 else (n // g2, g)


def dequant(N, K, g1, g2, g2_axis, codes, s_int, z1, s2, z2):
    """Matrix of Fractions Wd[n][k] (exact values of the half results)."""
    G = K // g1
    W = [[None] * K for _ in range(N)]
    for n in range(N):
        for g in range(G):
            r, c = second_order_pair(n, g, g2, g2_axis)
            s1 = scale_dequant(int(s_int[n][g]), int(z2[r][c]), int(s2[r][c]))
            for k in range(g * g1, (g + 1) * g1):
                W[n][k] = weight_dequant(int(codes[n][k]), int(z1[n][g]), s1)
    return W


def gemm(W, row_ptr, col, val, X_bits):
    """Exact rational product: dense part plus outlier part; Y[m][n] as Fractions."""
    N, K = len(W), len(W[0])
    M = len(X_bits)
    Y = [[Fraction(0)] * N for _ in range(M)]
    for m in range(M):
        x = [half_bits_to_fraction(int(b)) for b in X_bits[m]]
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                acc += W[n][k] * x[k]
            for e in range(int(row_ptr[n]), int(row_ptr[n + 1])):
                acc += half_bits_to_fraction(int(val[e])) * x[int(col[e])]
            Y[m][n] = acc
    return Y
