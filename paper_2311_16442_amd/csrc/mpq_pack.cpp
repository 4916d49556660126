// mpq_pack.cpp - host side of the library: validation of the logical format, the packed-blob
// builder (Sec. 3.3 "Memory Alignment": two code matrices with aligned, width-homogeneous vector
// units), blob inspection and the average-bit formulas (Sec. 2.2, Sec. 3.3, Sec. 4.2).
#include <math.h>
#include <stddef.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "../../include/mpq.h"
#include "mpq_format.h"

namespace {

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

bool desc_ok(const mpq_desc* d) {
  if (d->N <= 0 || d->K <= 0 || d->g1 <= 0 || d->g2 <= 0) return false;
  if (d->K % d->g1 != 0) return false;
  if (d->K > 65535) return false;  // 16-bit column index (Sec. 2.3)
  if (d->g2_axis != 0 && d->g2_axis != 1) return false;
  if (d->meta != MPQ_META_BYTES && d->meta != MPQ_META_PAPER) return false;
  return true;
}

// Fills every derived field of the header from the shape, the number of 4-bit groups and nnz.
mpq_status plan(const mpq_desc* d, int32_t n4, int64_t nnz, int64_t ocap, MpqHeader* h) {
  if (!desc_ok(d) || nnz < 0 || n4 < 0 || n4 > d->K / d->g1) return MPQ_ERR_SHAPE;
  if (ocap < 0 || ocap % 32 != 0 || ocap > (int64_t)MPQ_TILE_ROWS * d->K + 32) return MPQ_ERR_SHAPE;
  // a piece (the part of a 16-byte unit inside one group) must cover whole decode steps of 8 columns
  if (d->g1 != 16 && d->g1 != 32 && d->g1 != 64 && d->g1 != 128) return MPQ_ERR_UNSUPPORTED;
  if (d->meta == MPQ_META_PAPER && d->g1 != 16) return MPQ_ERR_UNSUPPORTED;  // Sec. 3.3: groups of 16
  // rows that share a second-order pair must not straddle 16-row tiles in an irregular way
  if (d->g2_axis == 1 && (d->g2 < MPQ_TILE_ROWS ? MPQ_TILE_ROWS % d->g2 != 0 : d->g2 % MPQ_TILE_ROWS != 0))
    return MPQ_ERR_UNSUPPORTED;
  memset(h, 0, sizeof(*h));
  h->magic = MPQ_MAGIC;
  h->version = MPQ_VERSION;
  h->N = d->N; h->K = d->K; h->g1 = d->g1; h->g2 = d->g2; h->g2_axis = d->g2_axis;
  h->G = d->K / d->g1;
  h->S = (h->G + d->g2 - 1) / d->g2;
  h->n4 = n4;
  h->n2 = h->G - n4;
  h->U2 = d->g1 >= 64 ? h->n2 * (d->g1 / 64) : (h->n2 + mpq_pu2(d->g1) - 1) / mpq_pu2(d->g1);
  h->U4 = d->g1 >= 32 ? h->n4 * (d->g1 / 32) : (h->n4 + mpq_pu4(d->g1) - 1) / mpq_pu4(d->g1);
  h->B2 = (h->U2 + MPQ_UNITS_PER_BLOCK - 1) / MPQ_UNITS_PER_BLOCK;
  h->B4 = (h->U4 + MPQ_UNITS_PER_BLOCK - 1) / MPQ_UNITS_PER_BLOCK;
  h->T = (d->N + MPQ_TILE_ROWS - 1) / MPQ_TILE_ROWS;
  h->nnz = nnz;
  h->meta = (uint64_t)d->meta;
  const uint64_t C = (uint64_t)h->B2 + h->B4;
  h->ocap = (uint64_t)ocap;
  // 16-bit offsets in the unit table
  if (32ull * (uint64_t)h->G > 0xFFFFull || (uint64_t)mpq_meta2_zero(h) > 0xFFFFull) return MPQ_ERR_UNSUPPORTED;
  if (d->meta == MPQ_META_PAPER) {
    if (mpq_p_entries(h) > 0xFFFFu) return MPQ_ERR_UNSUPPORTED;
    h->side_bytes = (uint64_t)mpq_p_off_outl(h) + MPQ_OTILE_HEAD + 4ull * (uint64_t)ocap;
  } else {
    h->side_bytes = 32ull * (h->G + 1) + mpq_meta2_bytes(h) + MPQ_OTILE_HEAD + 4ull * (uint64_t)ocap;
  }
  h->codes_off = align_up(h->side_bytes, 128);
  uint64_t tile_end = h->codes_off + C * MPQ_BLOCK_BYTES;
  if (ocap > 0 && ocap <= 65535) {
    h->oidx_off = align_up(tile_end, 64);
    tile_end = h->oidx_off + 32ull * ((uint64_t)h->B2 + 1);
  }
  h->tile_stride = align_up(tile_end, MPQ_SECTION_ALIGN);
  uint64_t off = MPQ_HEADER_BYTES;
  h->off_units = off; off = align_up(off + 8ull * mpq_pu2(d->g1) * 4 * C, MPQ_SECTION_ALIGN);
  h->off_tiles = off; off = align_up(off + (uint64_t)h->T * h->tile_stride, MPQ_SECTION_ALIGN);
  h->total_bytes = off;
  return MPQ_OK;
}

// Largest number of outliers in any 16-row tile, rounded up to a multiple of 32; -1 if row_ptr is
// not a monotone sequence starting at 0.
int64_t tile_capacity(const mpq_desc* d, const int32_t* row_ptr) {
  if (row_ptr[0] != 0) return -1;
  for (int64_t n = 0; n < d->N; ++n)
    if (row_ptr[n + 1] < row_ptr[n]) return -1;
  int64_t cap = 0;
  for (int64_t n0 = 0; n0 < d->N; n0 += MPQ_TILE_ROWS) {
    const int64_t n1 = n0 + MPQ_TILE_ROWS < d->N ? n0 + MPQ_TILE_ROWS : d->N;
    const int64_t c = (int64_t)row_ptr[n1] - row_ptr[n0];
    if (c > cap) cap = c;
  }
  return (cap + 31) / 32 * 32;
}

int32_t count4(const mpq_desc* d, const uint8_t* is4) {
  int32_t n4 = 0;
  for (int32_t g = 0; g < d->K / d->g1; ++g) n4 += is4[g] ? 1 : 0;
  return n4;
}

// ---- software fp16 (IEEE binary16, round to nearest even) for the host quantizer
float half_to_float(uint16_t hbits) {
  const uint32_t sign = (uint32_t)(hbits & 0x8000u) << 16;
  const uint32_t e = (hbits >> 10) & 0x1Fu, m = hbits & 0x3FFu;
  uint32_t f;
  if (e == 0) {
    if (m == 0) { f = sign; }
    else {  // subnormal: value m * 2^-24
      float v = (float)m * 5.9604644775390625e-08f;
      memcpy(&f, &v, 4);
      f |= sign;
    }
  } else if (e == 31) {
    f = sign | 0x7F800000u | (m << 13);
  } else {
    f = sign | ((e + 112u) << 23) | (m << 13);
  }
  float out;
  memcpy(&out, &f, 4);
  return out;
}

uint16_t float_to_half(float v) {
  uint32_t f;
  memcpy(&f, &v, 4);
  const uint16_t sign = (uint16_t)((f >> 16) & 0x8000u);
  const uint32_t a = f & 0x7FFFFFFFu;
  if (a >= 0x7F800000u) return (uint16_t)(sign | 0x7C00u | (a > 0x7F800000u ? 0x200u : 0u));  // inf / NaN
  if (a >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);  // rounds to 2^16 or above: infinity
  if (a < 0x33000001u) return sign;                          // at most half of the smallest subnormal
  const int32_t e = (int32_t)(a >> 23) - 127;
  uint32_t mant = (a & 0x7FFFFFu) | 0x800000u;  // 24 significant bits
  int shift = e >= -14 ? 13 : 13 + (-14 - e);   // bits dropped (normal: 13; subnormal: more)
  const uint32_t kept = mant >> shift, rest = mant & ((1u << shift) - 1u), halfway = 1u << (shift - 1);
  uint32_t r = kept;
  if (rest > halfway || (rest == halfway && (kept & 1u))) ++r;
  if (e >= -14) {
    // r has 11 bits (implicit one at bit 10) or carried to 12 bits; adding the exponent absorbs the carry
    return (uint16_t)(sign | (uint16_t)((((uint32_t)(e + 15) << 10) - 0x400u) + r));
  }
  return (uint16_t)(sign | (uint16_t)r);  // subnormal (a carry into bit 10 is the smallest normal)
}

// the decoder's two steps on the host (definition at the top of mpq.h): separate binary32 operations
uint16_t host_scale_dequant(uint8_t s_int, uint16_t z2, uint16_t s2) {
  volatile float t = (float)s_int - half_to_float(z2);
  volatile float u = t * half_to_float(s2);
  return float_to_half(u);
}

uint16_t host_weight_dequant(uint8_t code, uint8_t z1, uint16_t s1) {
  volatile float p = (float)((int)code - (int)z1) * half_to_float(s1);
  return float_to_half(p);
}

}  // namespace

// Used by the device entry points: a header is accepted only if it is exactly what the packer
// would have written for the shape it records.
mpq_status mpq_internal_check_header(const void* hdr_host, MpqHeader* out) {
  if (!hdr_host) return MPQ_ERR_NULL;
  MpqHeader h, want;
  memcpy(&h, hdr_host, sizeof(h));
  if (h.magic != MPQ_MAGIC || h.version != MPQ_VERSION) return MPQ_ERR_BLOB;
  if (h.meta > 1) return MPQ_ERR_BLOB;
  mpq_desc d = {h.N, h.K, h.g1, h.g2, h.g2_axis, (int32_t)h.meta};
  if (!desc_ok(&d)) return MPQ_ERR_BLOB;
  if (plan(&d, h.n4, h.nnz, (int64_t)h.ocap, &want) != MPQ_OK) return MPQ_ERR_BLOB;
  if (memcmp(&h, &want, offsetof(MpqHeader, is4_bits)) != 0) return MPQ_ERR_BLOB;
  int32_t set = 0;
  for (int32_t g = 0; g < (int32_t)MPQ_IS4_BITS; ++g)
    if (h.is4_bits[g / 8] >> (g % 8) & 1) {
      if (g >= h.G) return MPQ_ERR_BLOB;
      ++set;
    }
  if (set != (h.G <= (int32_t)MPQ_IS4_BITS ? h.n4 : 0)) return MPQ_ERR_BLOB;
  *out = h;
  return MPQ_OK;
}

bool mpq_internal_unit_words(const MpqHeader* h, uint32_t* words) {
  if (h->G > (int32_t)MPQ_IS4_BITS || h->g1 < 64 || h->meta != MPQ_META_BYTES) return false;
  const int32_t up2 = h->g1 / 64, up4 = h->g1 / 32;  // units per group in the 2-bit / 4-bit stream
  const int32_t nsub = mpq_nsub(h->g2);
  const uint32_t zero_word = (uint32_t)(h->G * 32) | (mpq_meta2_zero(h) << 16);
  const int32_t C = h->B2 + h->B4;
  for (int32_t u = 0; u < 4 * C; ++u) words[u] = zero_word;
  int32_t i2 = 0, i4 = 0;  // groups of each width seen so far = their index in the stream
  for (int32_t g = 0; g < h->G; ++g) {
    const bool four = h->is4_bits[g / 8] >> (g % 8) & 1;
    const int32_t si = four ? h->n2 + i4 : i2;  // stream index: 2-bit groups first
    const uint32_t m2off = h->g2_axis == 0 ? (uint32_t)((g / h->g2) * 64) : (uint32_t)(si * 4 * nsub);
    const uint32_t word = (uint32_t)(si * 32) | (m2off << 16);
    const int32_t up = four ? up4 : up2, first = four ? 4 * h->B2 + i4 * up4 : i2 * up2;
    for (int32_t k = 0; k < up; ++k) words[first + k] = word;
    if (four) ++i4; else ++i2;
  }
  return true;
}

extern "C" {

const char* mpq_status_str(mpq_status s) {
  switch (s) {
    case MPQ_OK: return "ok";
    case MPQ_ERR_NULL: return "null pointer";
    case MPQ_ERR_SHAPE: return "invalid shape";
    case MPQ_ERR_ALIGN: return "pointer not 16-byte aligned";
    case MPQ_ERR_CODE_RANGE: return "code out of range for its group's bit width";
    case MPQ_ERR_OUTLIER_IN_4BIT: return "outlier inside a 4-bit group";
    case MPQ_ERR_CSR: return "malformed CSR";
    case MPQ_ERR_BLOB: return "bad blob header";
    case MPQ_ERR_SIZE: return "buffer too small";
    case MPQ_ERR_UNSUPPORTED: return "format not supported by this build";
    case MPQ_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

double mpq_avg_bits(const mpq_desc* d, int32_t n4, int64_t nnz, int mode, int ns_bits) {
  if (!d || !desc_ok(d) || n4 < 0 || nnz < 0) return -1.0;
  const double G = (double)(d->K / d->g1);
  if (n4 > (int32_t)G) return -1.0;
  const double NK = (double)d->N * (double)d->K;
  if (mode == 0) {
    const double pairs = d->g2_axis == 0
                             ? (double)d->N * (double)(((int64_t)G + d->g2 - 1) / d->g2)
                             : (double)((d->N + d->g2 - 1) / d->g2) * G;
    const double triples = (double)(((int64_t)G - n4 + 2) / 3);
    const double meta1 = d->meta == MPQ_META_PAPER ? (double)d->N * (2.0 * triples + 1.0 * n4) : 2.0 * d->N * G;
    const double bytes = (double)d->N * ((G - n4) * d->g1 / 4.0 + n4 * d->g1 / 2.0)  // codes
                         + meta1                                                     // s_int, z1
                         + (d->meta == MPQ_META_PAPER ? 3.0 : 4.0) * pairs           // s2, z2
                         + 4.0 * (double)nnz + 4.0 * ((double)d->N + 1.0);           // CSR
    return 8.0 * bytes / NK;
  }
  if (mode == 1) {
    if (ns_bits <= 0) return -1.0;
    const double alpha = 1.0 - n4 / G;
    const double two_bit = 2.0 + (2.0 + ns_bits) / d->g1 + (ns_bits + 16.0) / ((double)d->g1 * d->g2);
    return alpha * two_bit + (1.0 - alpha) * 4.0 + (16.0 + 16.0 - 2.0) * (double)nnz / NK;
  }
  if (mode == 2) {
    // Sec. 3.3 "Memory Alignment" as storage: the zero points and scales of three 2-bit groups in one
    // 16-bit word (3 x 2-bit zeros + 4 + 3 + 3 bits of scales, "Scale Clipping"), the second-order
    // zero padded to whole bytes ("Zero Padding") next to the fp16 second-order scale.
    if (ns_bits <= 0) return -1.0;
    const double alpha = 1.0 - n4 / G;
    const double padded = 8.0 * ((ns_bits + 7) / 8);
    const double two_bit = 2.0 + 16.0 / (3.0 * d->g1) + (padded + 16.0) / ((double)d->g1 * d->g2);
    return alpha * two_bit + (1.0 - alpha) * 4.0 + (16.0 + 16.0 - 2.0) * (double)nnz / NK;
  }
  return -1.0;
}

mpq_status mpq_quantize_host(const mpq_desc* d, const float* W, int32_t n4, double p_o,
                             const mpq_logical_out* o, int64_t outlier_capacity, int64_t* nnz_out) {
  if (!d || !W || !o || !nnz_out) return MPQ_ERR_NULL;
  if (!o->is4 || !o->codes || !o->s_int || !o->z1 || !o->s2 || !o->z2 || !o->row_ptr) return MPQ_ERR_NULL;
  if (!desc_ok(d)) return MPQ_ERR_SHAPE;
  const int64_t N = d->N, K = d->K, g1 = d->g1, g2 = d->g2, G = K / g1;
  if (n4 < 0 || n4 > G || !(p_o >= 0.0 && p_o <= 1.0) || outlier_capacity < 0) return MPQ_ERR_SHAPE;
  // ---- Sec. 3.3, eq. 9 with a unit Hessian: the n4 most sensitive groups are 4-bit
  std::vector<double> S((size_t)G, 0.0);
  for (int64_t g = 0; g < G; ++g) {
    double acc = 0.0;
    for (int64_t n = 0; n < N; ++n)
      for (int64_t k = g * g1; k < (g + 1) * g1; ++k) acc += (double)W[n * K + k] * (double)W[n * K + k];
    S[(size_t)g] = acc;
  }
  std::vector<int32_t> order((size_t)G);
  for (int64_t g = 0; g < G; ++g) order[(size_t)g] = (int32_t)g;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return S[(size_t)a] > S[(size_t)b]; });
  memset(o->is4, 0, (size_t)G);
  for (int32_t r = 0; r < n4; ++r) o->is4[order[(size_t)r]] = 1;
  // ---- Sec. 4.3: outliers only inside 2-bit groups, largest magnitudes of each row
  std::vector<int32_t> cols2;
  for (int64_t k = 0; k < K; ++k)
    if (!o->is4[k / g1]) cols2.push_back((int32_t)k);
  const int64_t cnt = (int64_t)floor(p_o * (double)cols2.size() + 0.5);
  if (N * cnt > outlier_capacity) return MPQ_ERR_SIZE;
  if (N * cnt > 0 && (!o->col || !o->val)) return MPQ_ERR_NULL;
  std::vector<uint8_t> is_out((size_t)(N * K), 0);
  std::vector<int32_t> pick(cols2);
  o->row_ptr[0] = 0;
  for (int64_t n = 0; n < N; ++n) {
    const float* w = W + n * K;
    if (cnt > 0) {
      pick = cols2;
      std::stable_sort(pick.begin(), pick.end(), [&](int32_t a, int32_t b) { return fabs((double)w[a]) > fabs((double)w[b]); });
      for (int64_t r = 0; r < cnt; ++r) is_out[(size_t)(n * K + pick[(size_t)r])] = 1;
    }
    o->row_ptr[n + 1] = (int32_t)((n + 1) * cnt);
  }
  // ---- eq. 2: the scale of every (row, group) from the range of its non-outlier weights
  std::vector<double> sc((size_t)(N * G)), lo((size_t)(N * G));
  for (int64_t n = 0; n < N; ++n)
    for (int64_t g = 0; g < G; ++g) {
      double mn = INFINITY, mx = -INFINITY;
      for (int64_t k = g * g1; k < (g + 1) * g1; ++k)
        if (!is_out[(size_t)(n * K + k)]) {
          const double v = (double)W[n * K + k];
          mn = v < mn ? v : mn;
          mx = v > mx ? v : mx;
        }
      if (mn > mx) mn = mx = 0.0;  // every weight of the group is an outlier
      const double levels = o->is4[g] ? 15.0 : 3.0;
      double s = (mx - mn) / levels;
      if (s == 0.0) s = mn != 0.0 ? fabs(mn) : 1.0;
      sc[(size_t)(n * G + g)] = s;
      lo[(size_t)(n * G + g)] = mn;
    }
  // ---- second-order quantization of the scales to 8 bits, then the decoder's view of every scale
  const int64_t S2 = (G + g2 - 1) / g2, NB = (N + g2 - 1) / g2;
  const int64_t nblocks = d->g2_axis == 0 ? N * S2 : NB * G;
  std::vector<uint16_t> s1((size_t)(N * G));
  for (int64_t b = 0; b < nblocks; ++b) {
    int64_t n0, n1, ga, gb;
    if (d->g2_axis == 0) { n0 = b / S2; n1 = n0 + 1; ga = (b % S2) * g2; gb = ga + g2 < G ? ga + g2 : G; }
    else { n0 = (b / G) * g2; n1 = n0 + g2 < N ? n0 + g2 : N; ga = b % G; gb = ga + 1; }
    double smin = INFINITY, smax = -INFINITY;
    for (int64_t n = n0; n < n1; ++n)
      for (int64_t g = ga; g < gb; ++g) {
        const double s = sc[(size_t)(n * G + g)];
        smin = s < smin ? s : smin;
        smax = s > smax ? s : smax;
      }
    const double step = (smax - smin) / 255.0, floor_step = smax / 2047.0;  // |z2| <= 2047: exact in fp16
    const uint16_t s2h = float_to_half((float)(step > floor_step ? step : floor_step));
    const double s2f = (double)half_to_float(s2h), safe = s2f == 0.0 ? 1.0 : s2f;
    const uint16_t z2h = float_to_half((float)nearbyint(-smin / safe));
    const double z2f = (double)half_to_float(z2h);
    o->s2[b] = s2h;
    o->z2[b] = z2h;
    for (int64_t n = n0; n < n1; ++n)
      for (int64_t g = ga; g < gb; ++g) {
        double q = nearbyint(sc[(size_t)(n * G + g)] / safe) + z2f;
        q = q < 0.0 ? 0.0 : q > 255.0 ? 255.0 : q;
        o->s_int[n * G + g] = (uint8_t)q;
        s1[(size_t)(n * G + g)] = host_scale_dequant((uint8_t)q, z2h, s2h);
      }
  }
  // ---- eqs. 3-4 against the reconstructed scale; outliers carry what the dense code does not
  int64_t e = 0;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t g = 0; g < G; ++g) {
      const double levels = o->is4[g] ? 15.0 : 3.0;
      const uint16_t s1h = s1[(size_t)(n * G + g)];
      const double s1f = (double)half_to_float(s1h);
      const bool ok = s1f != 0.0;
      double z = 0.0;
      if (ok) {
        z = nearbyint(-lo[(size_t)(n * G + g)] / s1f);
        z = z < 0.0 ? 0.0 : z > levels ? levels : z;
      }
      o->z1[n * G + g] = (uint8_t)z;
      for (int64_t k = g * g1; k < (g + 1) * g1; ++k) {
        double c = 0.0;
        if (ok) {
          c = nearbyint((double)W[n * K + k] / s1f) + z;
          c = c < 0.0 ? 0.0 : c > levels ? levels : c;
        }
        o->codes[n * K + k] = (uint8_t)c;
        if (is_out[(size_t)(n * K + k)]) {
          const double wd = (double)half_to_float(host_weight_dequant((uint8_t)c, (uint8_t)z, s1h));
          o->col[e] = (uint16_t)k;
          o->val[e] = float_to_half((float)((double)W[n * K + k] - wd));
          ++e;
        }
      }
    }
  *nnz_out = e;
  return MPQ_OK;
}

mpq_status mpq_quantize_outlier_capacity(const mpq_desc* d, int32_t n4, double p_o, int64_t* capacity) {
  if (!d || !capacity) return MPQ_ERR_NULL;
  if (!desc_ok(d)) return MPQ_ERR_SHAPE;
  const int64_t G = d->K / d->g1;
  if (n4 < 0 || n4 > G || !(p_o >= 0.0 && p_o <= 1.0)) return MPQ_ERR_SHAPE;
  *capacity = (int64_t)d->N * (int64_t)floor(p_o * (double)((G - n4) * d->g1) + 0.5);
  return MPQ_OK;
}

mpq_status mpq_packed_size(const mpq_desc* d, const uint8_t* is4, const int32_t* row_ptr, size_t* bytes) {
  if (!d || !is4 || !row_ptr || !bytes) return MPQ_ERR_NULL;
  if (!desc_ok(d)) return MPQ_ERR_SHAPE;
  const int64_t ocap = tile_capacity(d, row_ptr);
  if (ocap < 0) return MPQ_ERR_CSR;
  MpqHeader h;
  mpq_status st = plan(d, count4(d, is4), row_ptr[d->N], ocap, &h);
  if (st != MPQ_OK) return st;
  *bytes = (size_t)h.total_bytes;
  return MPQ_OK;
}

mpq_status mpq_pack_host(const mpq_desc* d, const mpq_logical* w, void* blob_host, size_t bytes) {
  if (!d || !w || !blob_host) return MPQ_ERR_NULL;
  if (!w->is4 || !w->codes || !w->s_int || !w->z1 || !w->s2 || !w->z2 || !w->row_ptr) return MPQ_ERR_NULL;
  if (!desc_ok(d)) return MPQ_ERR_SHAPE;
  const int64_t N = d->N, K = d->K, g1 = d->g1;
  const int64_t G = K / g1;
  // ---- validation of the logical matrix, before anything is written
  const int64_t ocap = tile_capacity(d, w->row_ptr);
  if (ocap < 0) return MPQ_ERR_CSR;
  const int64_t nnz = w->row_ptr[N];
  if (nnz > 0 && (!w->col || !w->val)) return MPQ_ERR_NULL;
  MpqHeader h;
  mpq_status st = plan(d, count4(d, w->is4), nnz, ocap, &h);
  if (st != MPQ_OK) return st;
  if (bytes < h.total_bytes) return MPQ_ERR_SIZE;
  for (int64_t n = 0; n < N; ++n) {
    const uint8_t* row = w->codes + n * K;
    for (int64_t g = 0; g < G; ++g) {
      const uint8_t hi = w->is4[g] ? 15 : 3;
      for (int64_t k = g * g1; k < (g + 1) * g1; ++k)
        if (row[k] > hi) return MPQ_ERR_CODE_RANGE;
    }
    if (d->meta == MPQ_META_PAPER) {
      // ranges of the aligned packing: 2-bit zero points, 4-bit scales of which the second and third of
      // every triple of 2-bit groups fit 3 bits, 4-bit zero points and scales of 4-bit groups
      int64_t pos = 0;
      for (int64_t g = 0; g < G; ++g) {
        const uint8_t sv = w->s_int[n * G + g], zv = w->z1[n * G + g];
        if (w->is4[g]) {
          if (sv > 15 || zv > 15) return MPQ_ERR_CODE_RANGE;
        } else {
          if (zv > 3 || sv > (pos % 3 == 0 ? 15 : 7)) return MPQ_ERR_CODE_RANGE;
          ++pos;
        }
      }
    }
    for (int32_t e = w->row_ptr[n]; e < w->row_ptr[n + 1]; ++e) {
      if (w->col[e] >= K) return MPQ_ERR_CSR;
      if (e > w->row_ptr[n] && w->col[e] <= w->col[e - 1]) return MPQ_ERR_CSR;
      if (w->is4[w->col[e] / g1]) return MPQ_ERR_OUTLIER_IN_4BIT;  // Sec. 4.3: only in 2-bit groups
    }
  }
  if (d->meta == MPQ_META_PAPER) {
    const int64_t pairs = d->g2_axis == 0 ? N * h.S : ((N + d->g2 - 1) / d->g2) * G;
    for (int64_t e = 0; e < pairs; ++e) {
      const float z = half_to_float(w->z2[e]);
      if (!(z >= 0.0f && z <= 15.0f) || z != (float)(int)z) return MPQ_ERR_CODE_RANGE;  // an Ns-bit integer
    }
  }
  // ---- layout
  uint8_t* blob = (uint8_t*)blob_host;
  memset(blob, 0, (size_t)h.total_bytes);
  if (G <= (int64_t)MPQ_IS4_BITS)
    for (int64_t g = 0; g < G; ++g)
      if (w->is4[g]) h.is4_bits[g / 8] |= (uint8_t)(1u << (g % 8));
  memcpy(blob, &h, sizeof(h));
  // stream order of the groups and the unit tables
  std::vector<int32_t> groups2, groups4, stream_index(G);
  for (int32_t g = 0; g < G; ++g) (w->is4[g] ? groups4 : groups2).push_back(g);
  for (size_t i = 0; i < groups2.size(); ++i) stream_index[groups2[i]] = (int32_t)i;
  for (size_t i = 0; i < groups4.size(); ++i) stream_index[groups4[i]] = (int32_t)(h.n2 + i);
  // pieces: for every unit slot the K-group it decodes (-1 = padding) and its first column
  const int32_t PU2 = mpq_pu2(d->g1), PU4 = mpq_pu4(d->g1);
  const int32_t cpp2 = g1 >= 64 ? 64 : (int32_t)g1, cpp4 = g1 >= 32 ? 32 : (int32_t)g1;  // columns per piece
  const int32_t nsub = mpq_nsub(d->g2);
  const uint32_t zero_word1 = (uint32_t)(G * 32) | (mpq_meta2_zero(&h) << 16);
  const int64_t nunits = 4ll * (h.B2 + h.B4);
  std::vector<int32_t> piece_g((size_t)nunits * PU2, -1);
  std::vector<int64_t> piece_k0((size_t)nunits * PU2, 0);
  for (int64_t u = 0; u < nunits; ++u) {
    const bool four = u >= 4ll * h.B2;
    const int64_t ul = four ? u - 4ll * h.B2 : u;
    const std::vector<int32_t>& groups = four ? groups4 : groups2;
    const int32_t PU = four ? PU4 : PU2, cpp = four ? cpp4 : cpp2;
    if (ul >= (four ? h.U4 : h.U2)) continue;
    for (int32_t q = 0; q < PU; ++q) {
      int64_t gi, koff;
      if (g1 >= (four ? 32 : 64)) { const int64_t upg = g1 / cpp; gi = ul / upg; koff = cpp * (ul % upg); }
      else { gi = ul * PU + q; koff = 0; }
      if (gi >= (int64_t)groups.size()) continue;
      piece_g[(size_t)(u * PU2 + q)] = groups[(size_t)gi];
      piece_k0[(size_t)(u * PU2 + q)] = (int64_t)groups[(size_t)gi] * g1 + koff;
    }
  }
  uint32_t* unit_tab = (uint32_t*)(blob + h.off_units);
  for (int64_t p = 0; p < nunits * PU2; ++p) {
    const int32_t g = piece_g[(size_t)p];
    if (d->meta == MPQ_META_PAPER) {
      // word 1: offset of the triple (+ position in it) or of the 4-bit group | first second-order entry << 16
      const bool four = p >= 4ll * h.B2 * PU2;
      if (g < 0) {
        unit_tab[2 * p] = 0;
        unit_tab[2 * p + 1] = (four ? 16u * (uint32_t)h.n4 : 32u * mpq_p_triples(&h)) | (mpq_p_zero_entry(&h) << 16);
        continue;
      }
      const uint32_t si = (uint32_t)stream_index[g];
      const uint32_t m1 = four ? 16u * (si - (uint32_t)h.n2) : 32u * (si / 3u) + si % 3u;
      const uint32_t e2 = d->g2_axis == 0 ? (uint32_t)(g / d->g2) * 16u : si * (uint32_t)nsub;
      unit_tab[2 * p] = (uint32_t)(2 * piece_k0[(size_t)p]);
      unit_tab[2 * p + 1] = m1 | (e2 << 16);
      continue;
    }
    if (g < 0) { unit_tab[2 * p] = 0; unit_tab[2 * p + 1] = zero_word1; continue; }
    const uint32_t m2off = d->g2_axis == 0 ? (uint32_t)((g / d->g2) * 64) : (uint32_t)(stream_index[g] * 4 * nsub);
    unit_tab[2 * p] = (uint32_t)(2 * piece_k0[(size_t)p]);
    unit_tab[2 * p + 1] = (uint32_t)(stream_index[g] * 32) | (m2off << 16);
  }
  const uint64_t m2_bytes = mpq_meta2_bytes(&h);
  for (int64_t n = 0; n < N; ++n) {
    const int64_t t = n / MPQ_TILE_ROWS, i = n % MPQ_TILE_ROWS;
    uint8_t* tile = blob + h.off_tiles + (uint64_t)t * h.tile_stride;
    uint16_t* meta1 = (uint16_t*)tile;
    uint32_t* meta2 = (uint32_t*)(tile + 32ull * (G + 1));
    uint32_t* codes = (uint32_t*)(tile + h.codes_off);
    const uint8_t* row = w->codes + n * K;
    for (int64_t u = 0; u < nunits; ++u) {
      const bool four = u >= 4ll * h.B2;
      const int32_t PU = four ? PU4 : PU2, cpp = four ? cpp4 : cpp2;
      uint32_t* q4 = codes + (((u / 4) * 64 + (u % 4) * 16 + i) * 4);
      for (int32_t q = 0; q < PU; ++q) {
        if (piece_g[(size_t)(u * PU2 + q)] < 0) continue;
        const int64_t k0 = piece_k0[(size_t)(u * PU2 + q)];
        for (int32_t kp = 0; kp < cpp; ++kp) {
          const int32_t kl = q * cpp + kp;  // column inside the unit
          const uint32_t code = row[k0 + kp];
          uint32_t& dw = q4[(kl % 8) / 2];
          if (four) {
            dw |= code << (16 * (kl % 2) + 4 * (kl / 8));
          } else {
            // decode step P = kl / 8; nibble (P % 4) + 4 * (kl % 2) of the dword (see mpq_format.h)
            const int32_t nn = (kl / 8) % 4 + 4 * (kl % 2);
            if (kl < 32) dw |= code << (4 * nn + 1);
            else dw |= ((code & 1u) << (4 * nn + 3)) | ((code >> 1) << ((4 * nn + 4) % 32));
          }
        }
      }
    }
    if (d->meta == MPQ_META_PAPER) {
      uint8_t* m1b = tile + mpq_p_off_m1b(&h);
      uint16_t* s2a = (uint16_t*)(tile + mpq_p_off_s2(&h));
      uint8_t* z2a = tile + mpq_p_off_z2(&h);
      for (int64_t g = 0; g < G; ++g) {
        const uint32_t si = (uint32_t)stream_index[g], sv = w->s_int[n * G + g], zv = w->z1[n * G + g];
        if (w->is4[g]) {
          m1b[(si - (uint32_t)h.n2) * MPQ_TILE_ROWS + i] = (uint8_t)(sv | (zv << 4));
        } else {
          const uint32_t pos = si % 3u;  // zero points at bits 0-5, scales at bits 6 (4 bits), 10 and 13 (3 bits)
          meta1[(si / 3u) * MPQ_TILE_ROWS + i] |= (uint16_t)((zv << (2u * pos)) | (sv << (pos == 0 ? 6u : pos == 1 ? 10u : 13u)));
        }
      }
      // the second-order zero as the integer it is (validated below to be one), in a byte
      auto z2_byte = [&](uint16_t zbits) { return (uint8_t)half_to_float(zbits); };
      if (d->g2_axis == 0) {
        for (int64_t s2i = 0; s2i < h.S; ++s2i) {
          s2a[s2i * MPQ_TILE_ROWS + i] = w->s2[n * h.S + s2i];
          z2a[s2i * MPQ_TILE_ROWS + i] = z2_byte(w->z2[n * h.S + s2i]);
        }
      } else if (i % d->g2 == 0 || (d->g2 >= MPQ_TILE_ROWS && i == 0)) {
        const int64_t nb = n / d->g2, sub = d->g2 >= MPQ_TILE_ROWS ? 0 : i / d->g2;
        for (int64_t g = 0; g < G; ++g) {
          s2a[stream_index[g] * nsub + sub] = w->s2[nb * G + g];
          z2a[stream_index[g] * nsub + sub] = z2_byte(w->z2[nb * G + g]);
        }
      }
      continue;
    }
    for (int64_t g = 0; g < G; ++g)
      meta1[stream_index[g] * MPQ_TILE_ROWS + i] = (uint16_t)(w->s_int[n * G + g] | ((uint16_t)w->z1[n * G + g] << 8));
    if (d->g2_axis == 0) {
      for (int64_t s2i = 0; s2i < h.S; ++s2i)
        meta2[s2i * MPQ_TILE_ROWS + i] = (uint32_t)w->s2[n * h.S + s2i] | ((uint32_t)w->z2[n * h.S + s2i] << 16);
    } else if (i % d->g2 == 0 || (d->g2 >= MPQ_TILE_ROWS && i == 0)) {
      // first row of a block of g2 rows inside the tile: the block's pair for every group
      const int64_t nb = n / d->g2, sub = d->g2 >= MPQ_TILE_ROWS ? 0 : i / d->g2;
      for (int64_t g = 0; g < G; ++g)
        meta2[stream_index[g] * nsub + sub] = (uint32_t)w->s2[nb * G + g] | ((uint32_t)w->z2[nb * G + g] << 16);
    }
  }
  (void)m2_bytes;
  for (int64_t t = 0; t < h.T; ++t) {
    const uint64_t off_outl = d->meta == MPQ_META_PAPER ? (uint64_t)mpq_p_off_outl(&h) : 32ull * (G + 1) + mpq_meta2_bytes(&h);
    uint32_t* rec = (uint32_t*)(blob + h.off_tiles + (uint64_t)t * h.tile_stride + off_outl);
    const int64_t n0 = t * MPQ_TILE_ROWS;
    const int32_t base = w->row_ptr[n0];
    for (int r = 0; r <= MPQ_TILE_ROWS; ++r) {
      const int64_t n = n0 + r < N ? n0 + r : N;
      rec[r] = (uint32_t)(w->row_ptr[n] - base);
    }
    const int64_t nend = n0 + MPQ_TILE_ROWS < N ? n0 + MPQ_TILE_ROWS : N;
    uint32_t* words = rec + MPQ_OTILE_HEAD / 4;
    for (int32_t e = base; e < w->row_ptr[nend]; ++e)
      words[e - base] = (uint32_t)w->col[e] | ((uint32_t)w->val[e] << 16);
    if (h.oidx_off) {
      // the 2-bit block of a column follows from its group's place in the 2-bit stream: g1 / 64 units per group, or
      // PU2 groups per unit
      uint16_t* oidx = (uint16_t*)(blob + h.off_tiles + (uint64_t)t * h.tile_stride + h.oidx_off);
      const int64_t upg = g1 / 64;
      for (int r = 0; r < MPQ_TILE_ROWS; ++r) {
        const int64_t n = n0 + r < N ? n0 + r : N;
        const int64_t n1 = n0 + r + 1 < N ? n0 + r + 1 : N;
        int32_t e = w->row_ptr[n];
        for (int64_t c = 0; c <= h.B2; ++c) {
          while (e < w->row_ptr[n1]) {
            const int64_t k = w->col[e], g = k / g1;
            const int64_t unit = g1 >= 64 ? (int64_t)stream_index[g] * upg + (k % g1) / 64 : (int64_t)stream_index[g] / PU2;
            const int64_t blk = unit / MPQ_UNITS_PER_BLOCK;
            if (blk >= c) break;
            ++e;
          }
          oidx[c * MPQ_TILE_ROWS + r] = (uint16_t)((c == h.B2 ? w->row_ptr[n1] : e) - base);
        }
      }
    }
  }
  return MPQ_OK;
}

mpq_status mpq_blob_info(const void* hdr_host, mpq_desc* out, int64_t* nnz, int32_t* n4,
                         uint64_t* total_bytes) {
  if (!hdr_host) return MPQ_ERR_NULL;
  MpqHeader h;
  memcpy(&h, hdr_host, sizeof(h));
  if (h.magic != MPQ_MAGIC || h.version != MPQ_VERSION) return MPQ_ERR_BLOB;
  if (out) { out->N = h.N; out->K = h.K; out->g1 = h.g1; out->g2 = h.g2; out->g2_axis = h.g2_axis; out->meta = (int32_t)h.meta; }
  if (nnz) *nnz = h.nnz;
  if (n4) *n4 = h.n4;
  if (total_bytes) *total_bytes = h.total_bytes;
  return MPQ_OK;
}

mpq_status mpq_blob_tiles(const void* hdr_host, uint64_t* first_offset, uint64_t* record_bytes, int32_t* count) {
  if (!hdr_host || !first_offset || !record_bytes || !count) return MPQ_ERR_NULL;
  MpqHeader h;
  const mpq_status st = mpq_internal_check_header(hdr_host, &h);
  if (st != MPQ_OK) return st;
  *first_offset = h.off_tiles;
  *record_bytes = h.tile_stride;
  *count = h.T;
  return MPQ_OK;
}

}  // extern "C"
