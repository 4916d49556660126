/*
 * mpq_oracle.c - plain CPU reference ("oracle") for the 2/4/16-bit mixed-precision weight format
 * of arXiv 2311.16442.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the HIP library can be checked against an
 * independent, slow, obviously correct implementation.  Only the test-suite, the smoke check and
 * the benchmark's CPU-baseline leg may call it; the product never does.  It shares no code, table
 * or header with the HIP path and reads the *logical* (unpacked) arrays, never the packed blob.
 *
 * What it computes is a definition, not an approximation, so it is the definition written out:
 *
 *   second-order dequantization of the scale   (Sec. 3.3; Algorithm 1, second-order dequantization
 *                                               step; eq. 5 form (q - z) * s)
 *       t  = fp32(s_int) - fp32(z2)            one binary32 subtraction
 *       u  = t * fp32(s2)                      one binary32 multiplication (not fused with the above)
 *       s1 = fp16(u)                           the scaling factor is a half (Sec. 2.2)
 *   first-order dequantization of the weight   (Sec. 2.2 eq. 5; Algorithm 1, first-order dequantization
 *                                               step; weights restored to half, Sec. 5.1)
 *       d  = code - z1                         exact integer
 *       Wd = fp16(fp32(d) * fp32(s1))          exact product, one rounding
 *   outliers are a separate fp16 sparse matrix added to the dense one (Sec. 2.3, Sec. 4.1)
 *       Wfull = fp16(fp32(Wd) + fp32(val))     at CSR positions
 *   product (Algorithm 1, the accumulation step, then the sparse product added, Sec. 4.1)
 *       y[m][n] = sum_k (double)Wd[n][k] * (double)X[m][k]  +  sum_j (double)val_j * (double)X[m][col_j]
 *     accumulated in binary64, k ascending, outliers after the dense part.
 *
 * All conversions are IEEE 754 round-to-nearest-even with gradual underflow, written out in
 * software below (no compiler half type, no hardware conversion instruction).
 *
 * Readings of points the paper leaves open (each listed in the design notes of the repository):
 *   - only the scale is second-order quantized; the first-order zero point is an integer used as is;
 *   - the second-order pair covers g2 consecutive K-groups of a row (g2_axis 0, what the benchmark
 *     configurations state) or the same K-group of g2 consecutive rows (g2_axis 1, the paper's
 *     wording: along the output channels);
 *   - the last second-order group is short when G is not a multiple of g2 (resp. N for axis 1).
 *
 * Pins (tests/test_oracle_*.py): exact rational brute force with independent rounding on tiny
 * matrices; numpy's IEEE half type for every conversion; integer and CSR special cases; the
 * average-bit values printed in the paper.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ fp16 <-> fp32, in software */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* binary16 -> binary32, exact. */
float orc_half_to_float(uint16_t h) {
  uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  uint32_t exp = (h >> 10) & 0x1Fu;
  uint32_t man = h & 0x3FFu;
  if (exp == 0x1Fu) return bits_f32(sign | 0x7F800000u | (man << 13));   /* inf / nan */
  if (exp == 0) {
    if (man == 0) return bits_f32(sign);                                  /* +-0 */
    /* subnormal: value = man * 2^-24; normalise */
    int e = -1;
    do { man <<= 1; ++e; } while ((man & 0x400u) == 0);
    man &= 0x3FFu;
    return bits_f32(sign | ((uint32_t)(127 - 15 - e) << 23) | (man << 13));
  }
  return bits_f32(sign | ((exp + 127 - 15) << 23) | (man << 13));
}

/* binary32 -> binary16, round to nearest, ties to even, gradual underflow, overflow to inf. */
uint16_t orc_float_to_half(float f) {
  uint32_t u = f32_bits(f);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  uint32_t exp = (u >> 23) & 0xFFu;
  uint32_t man = u & 0x7FFFFFu;
  if (exp == 0xFFu) {                                  /* inf or nan */
    if (man == 0) return (uint16_t)(sign | 0x7C00u);
    return (uint16_t)(sign | 0x7E00u | (man >> 13));   /* quiet nan, keep top payload bits */
  }
  int e = (int)exp - 127;                              /* unbiased exponent of 1.m */
  if (e > 15) return (uint16_t)(sign | 0x7C00u);       /* too large even before rounding */
  if (e >= -14) {                                      /* normal half (may round up into the next binade/inf) */
    uint32_t half_exp = (uint32_t)(e + 15);
    uint32_t keep = man >> 13;
    uint32_t rest = man & 0x1FFFu;
    uint32_t out = (half_exp << 10) | keep;
    if (rest > 0x1000u || (rest == 0x1000u && (out & 1u))) out += 1;   /* carry may ripple into exponent: correct */
    return (uint16_t)(sign | out);
  }
  /* result is subnormal or zero: value = 1.m * 2^e, unit of half subnormals is 2^-24 */
  if (e < -25) return sign;                            /* below half of the smallest subnormal -> 0 (e == -25 handled below) */
  uint32_t full = man | 0x800000u;                     /* 24-bit significand, value = full * 2^(e-23) */
  int shift = (-24) - (e - 23);                        /* want units of 2^-24: full >> shift */
  /* shift is between 14 (e = -15) and 24 (e = -25) */
  uint32_t keep = full >> shift;
  uint32_t rest = full & ((1u << shift) - 1u);
  uint32_t halfway = 1u << (shift - 1);
  if (rest > halfway || (rest == halfway && (keep & 1u))) keep += 1;   /* may become 0x400 = smallest normal: correct */
  return (uint16_t)(sign | keep);
}

/* ------------------------------------------------------------------ the two dequantizations */

/* Second-order dequantization of one first-order scale (Algorithm 1; eq. 5 form). */
uint16_t orc_scale_dequant(uint8_t s_int, uint16_t z2, uint16_t s2) {
  volatile float t = (float)s_int - orc_half_to_float(z2);
  volatile float u = t * orc_half_to_float(s2);
  return orc_float_to_half(u);
}

/* First-order dequantization of one weight (eq. 5). */
uint16_t orc_weight_dequant(uint8_t code, uint8_t z1, uint16_t s1) {
  int d = (int)code - (int)z1;
  volatile float p = (float)d * orc_half_to_float(s1);
  return orc_float_to_half(p);
}

/* Sum of a dequantized weight and an outlier value, both half (dense + sparse matrix, Sec. 2.3). */
uint16_t orc_add_outlier(uint16_t w, uint16_t val) {
  volatile float s = orc_half_to_float(w) + orc_half_to_float(val);
  return orc_float_to_half(s);
}

typedef struct {
  int32_t N, K, g1, g2, g2_axis;
} orc_desc;

static int64_t second_order_index(const orc_desc* d, int64_t n, int64_t g) {
  int64_t G = d->K / d->g1;
  if (d->g2_axis == 0) {
    int64_t S = (G + d->g2 - 1) / d->g2;
    return n * S + g / d->g2;
  }
  return (n / d->g2) * G + g;
}

/* Checks of the logical format; returns 0 when valid, else a positive code:
 * 1 shape, 2 code out of range, 3 CSR malformed, 4 outlier inside a 4-bit group. */
int orc_validate(const orc_desc* d, const uint8_t* is4, const uint8_t* codes,
                 const int32_t* row_ptr, const uint16_t* col) {
  if (d->N <= 0 || d->K <= 0 || d->g1 <= 0 || d->g2 <= 0 || d->K % d->g1 != 0 || d->K > 65535) return 1;
  for (int64_t n = 0; n < d->N; ++n)
    for (int64_t k = 0; k < d->K; ++k) {
      int hi = is4[k / d->g1] ? 15 : 3;
      if (codes[n * d->K + k] > hi) return 2;
    }
  if (row_ptr[0] != 0) return 3;
  for (int64_t n = 0; n < d->N; ++n) {
    if (row_ptr[n + 1] < row_ptr[n]) return 3;
    for (int32_t j = row_ptr[n]; j < row_ptr[n + 1]; ++j) {
      if (col[j] >= d->K) return 3;
      if (j > row_ptr[n] && col[j] <= col[j - 1]) return 3;
      if (is4[col[j] / d->g1]) return 4;
    }
  }
  return 0;
}

/* First-order scales of the whole matrix: s1_out[n*G + g] (half bits). */
void orc_scales(const orc_desc* d, const uint8_t* s_int, const uint16_t* s2, const uint16_t* z2,
                uint16_t* s1_out) {
  int64_t G = d->K / d->g1;
  for (int64_t n = 0; n < d->N; ++n)
    for (int64_t g = 0; g < G; ++g) {
      int64_t j = second_order_index(d, n, g);
      s1_out[n * G + g] = orc_scale_dequant(s_int[n * G + g], z2[j], s2[j]);
    }
}

/* Dense dequantization Wd (add_outliers = 0) or dense + sparse Wfull (add_outliers = 1),
 * row-major N x K half bits. */
void orc_dequant(const orc_desc* d, const uint8_t* codes, const uint8_t* s_int, const uint8_t* z1,
                 const uint16_t* s2, const uint16_t* z2, const int32_t* row_ptr, const uint16_t* col,
                 const uint16_t* val, int add_outliers, uint16_t* W_out) {
  int64_t G = d->K / d->g1;
  for (int64_t n = 0; n < d->N; ++n) {
    for (int64_t g = 0; g < G; ++g) {
      int64_t j = second_order_index(d, n, g);
      uint16_t s1 = orc_scale_dequant(s_int[n * G + g], z2[j], s2[j]);
      for (int64_t k = g * d->g1; k < (g + 1) * d->g1; ++k)
        W_out[n * d->K + k] = orc_weight_dequant(codes[n * d->K + k], z1[n * G + g], s1);
    }
    if (add_outliers)
      for (int32_t e = row_ptr[n]; e < row_ptr[n + 1]; ++e) {
        int64_t at = n * d->K + col[e];
        W_out[at] = orc_add_outlier(W_out[at], val[e]);
      }
  }
}

/* Y[m*N + n] (binary64) = dense product + outlier product, for rows n in [n_begin, n_end).
 * X is M x K half bits, row-major.  `threads` > 1 splits the rows over that many OpenMP threads
 * (each output is still one sequential binary64 sum, so the result does not depend on `threads`). */
void orc_gemm_rows(const orc_desc* d, const uint8_t* codes, const uint8_t* s_int, const uint8_t* z1,
                   const uint16_t* s2, const uint16_t* z2, const int32_t* row_ptr, const uint16_t* col,
                   const uint16_t* val, const uint16_t* X, int32_t M, int64_t n_begin, int64_t n_end,
                   int threads, double* Y) {
  int64_t G = d->K / d->g1;
  int64_t K = d->K;
  (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads > 1 ? threads : 1)
#endif
  for (int64_t n = n_begin; n < n_end; ++n) {
    double* xrow = (double*)malloc(sizeof(double) * (size_t)K);
    double* wrow = (double*)malloc(sizeof(double) * (size_t)K);
    for (int64_t g = 0; g < G; ++g) {
      int64_t j = second_order_index(d, n, g);
      uint16_t s1 = orc_scale_dequant(s_int[n * G + g], z2[j], s2[j]);
      for (int64_t k = g * d->g1; k < (g + 1) * d->g1; ++k)
        wrow[k] = (double)orc_half_to_float(orc_weight_dequant(codes[n * K + k], z1[n * G + g], s1));
    }
    for (int32_t m = 0; m < M; ++m) {
      for (int64_t k = 0; k < K; ++k) xrow[k] = (double)orc_half_to_float(X[(int64_t)m * K + k]);
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) acc += wrow[k] * xrow[k];
      for (int32_t e = row_ptr[n]; e < row_ptr[n + 1]; ++e)
        acc += (double)orc_half_to_float(val[e]) * xrow[col[e]];
      Y[(int64_t)m * d->N + n] = acc;
    }
    free(xrow);
    free(wrow);
  }
}

/* ------------------------------------------------------------------ average bits per weight */

/* Sec. 2.2, first case of the average-bit display: N-bit codes, N-bit zero and 16-bit scale per group. */
double orc_avg_bits_first_order(int nbits, int g1) { return nbits + (nbits + 16.0) / g1; }

/* Sec. 2.2, second case: Ns-bit scale, N-bit zero per group; Ns-bit zero and 16-bit scale per g2 groups. */
double orc_avg_bits_second_order(int nbits, int ns, int g1, int g2) {
  return nbits + (double)(nbits + ns) / g1 + (ns + 16.0) / ((double)g1 * g2);
}

/* Sec. 3.3: alpha = share of 2-bit groups; 4-bit groups are charged exactly 4 bits as printed. */
double orc_avg_bits_mixed(double alpha, int ns, int g1, int g2) {
  return alpha * orc_avg_bits_second_order(2, ns, g1, g2) + (1.0 - alpha) * 4.0;
}

/* Sec. 4.2: each outlier costs 16 (value) + 16 (index) bits and frees its 2-bit code. */
double orc_outlier_bits(double ratio) { return (16.0 + 16.0 - 2.0) * ratio; }

/* Bits per weight this format really stores: codes at 2 or 4 bits, one byte each of s_int and z1
 * per (row, group), two halves per (row, second-order group), 32 bits per outlier and per row pointer. */
double orc_avg_bits_stored(const orc_desc* d, int32_t n4, int64_t nnz) {
  double G = (double)(d->K / d->g1);
  double S = d->g2_axis == 0 ? (double)((d->K / d->g1 + d->g2 - 1) / d->g2) * d->N
                             : (double)((d->N + d->g2 - 1) / d->g2) * G;
  double NK = (double)d->N * d->K;
  double code_bits = (double)d->N * d->g1 * (2.0 * (G - n4) + 4.0 * n4);
  double meta_bits = 16.0 * d->N * G + 32.0 * S;
  double csr_bits = 32.0 * (double)nnz + 32.0 * ((double)d->N + 1.0);
  return (code_bits + meta_bits + csr_bits) / NK;
}

/* ------------------------------------------------------------------ aligned metadata (Sec. 3.3 "Memory Alignment")
 *
 * The paper packs the zero points and scales of three 2-bit groups of 16 weights into one 16-bit word:
 * 3 x 2 bits of zero points, one scale of Ns = 4 bits and two scales held in 3 bits
 * (Scale Clipping); the second-order zero is an Ns-bit integer stored padded.  Which two
 * scales lose a bit, and how, is not stated.  Reading taken here (and by the library): count a row's 2-bit
 * groups in K order; in every run of three the first keeps 4 bits, the second and third are clipped
 * (saturated) to 3 bits, i.e. to at most 7.  4-bit groups (about which the paper says nothing) keep a
 * 4-bit scale and a 4-bit zero point.  The decode formula is unchanged: it is applied to the values as
 * stored. */

/* What a quantizer that targets the aligned format does to 4-bit scale codes: s_out = s_in, clipped to 7
 * where the format has only 3 bits, to 15 elsewhere. */
void orc_clip_scales(const orc_desc* d, const uint8_t* is4, const uint8_t* s_in, uint8_t* s_out) {
  int64_t G = d->K / d->g1;
  for (int64_t n = 0; n < d->N; ++n) {
    int64_t seen2 = 0; /* 2-bit groups of this row so far */
    for (int64_t g = 0; g < G; ++g) {
      int limit = 15;
      if (!is4[g]) {
        if (seen2 % 3 != 0) limit = 7;
        ++seen2;
      }
      s_out[n * G + g] = s_in[n * G + g] > limit ? (uint8_t)limit : s_in[n * G + g];
    }
  }
}

/* 0 if the logical arrays fit the aligned format, else 5: a zero point beyond its group's bit width, a
 * scale beyond its field, or a second-order zero that is not an integer 0..15. */
int orc_validate_aligned(const orc_desc* d, const uint8_t* is4, const uint8_t* s_int, const uint8_t* z1,
                         const uint16_t* z2) {
  int64_t G = d->K / d->g1;
  for (int64_t n = 0; n < d->N; ++n) {
    int64_t seen2 = 0;
    for (int64_t g = 0; g < G; ++g) {
      if (is4[g]) {
        if (s_int[n * G + g] > 15 || z1[n * G + g] > 15) return 5;
      } else {
        if (z1[n * G + g] > 3 || s_int[n * G + g] > (seen2 % 3 == 0 ? 15 : 7)) return 5;
        ++seen2;
      }
    }
  }
  int64_t pairs = d->g2_axis == 0 ? (int64_t)d->N * ((G + d->g2 - 1) / d->g2) : (int64_t)((d->N + d->g2 - 1) / d->g2) * G;
  for (int64_t e = 0; e < pairs; ++e) {
    float z = orc_half_to_float(z2[e]);
    if (!(z >= 0.0f && z <= 15.0f) || z != (float)(int)z) return 5;
  }
  return 0;
}

/* Bits per weight the aligned format stores: codes; 16 bits per (row, three 2-bit groups, the last run
 * of a row possibly short); 8 bits per (row, 4-bit group); 16 + 8 bits per second-order pair; CSR. */
double orc_avg_bits_stored_aligned(const orc_desc* d, int32_t n4, int64_t nnz) {
  int64_t G = d->K / d->g1, n2 = G - n4;
  double pairs = d->g2_axis == 0 ? (double)d->N * (double)((G + d->g2 - 1) / d->g2)
                                 : (double)((d->N + d->g2 - 1) / d->g2) * (double)G;
  double NK = (double)d->N * d->K;
  double code_bits = (double)d->N * d->g1 * (2.0 * n2 + 4.0 * n4);
  double meta_bits = (double)d->N * (16.0 * (double)((n2 + 2) / 3) + 8.0 * n4) + 24.0 * pairs;
  double csr_bits = 32.0 * (double)nnz + 32.0 * ((double)d->N + 1.0);
  return (code_bits + meta_bits + csr_bits) / NK;
}

int orc_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
