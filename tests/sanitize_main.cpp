// Host-only exercise of the packer, the reference quantizer and the CPU oracle for a build with
// -fsanitize=address,undefined (see test_host_sanitizers.py): random small matrices in every supported
// group size and both second-order axes, malformed inputs that must be refused, and the oracle's
// decode and product on the same data.  Exit status 0 = every call behaved and the sanitizers stayed silent.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <random>
#include <vector>

#include "../include/mpq.h"

extern "C" {
typedef struct { int32_t N, K, g1, g2, g2_axis; } orc_desc;
int orc_validate(const orc_desc* d, const uint8_t* is4, const uint8_t* codes, const int32_t* row_ptr, const uint16_t* col);
void orc_dequant(const orc_desc* d, const uint8_t* codes, const uint8_t* s_int, const uint8_t* z1, const uint16_t* s2,
                 const uint16_t* z2, const int32_t* row_ptr, const uint16_t* col, const uint16_t* val, int add_outliers,
                 uint16_t* W_out);
void orc_gemm_rows(const orc_desc* d, const uint8_t* codes, const uint8_t* s_int, const uint8_t* z1, const uint16_t* s2,
                   const uint16_t* z2, const int32_t* row_ptr, const uint16_t* col, const uint16_t* val, const uint16_t* X,
                   int32_t M, int64_t n_begin, int64_t n_end, int threads, double* Y);
uint16_t orc_float_to_half(float f);
double orc_avg_bits_stored(const orc_desc* d, int32_t n4, int64_t nnz);
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static int one(int N, int K, int g1, int g2, int axis, double f4, double p_o, unsigned seed) {
  std::mt19937 rng(seed);
  const int G = K / g1, n4 = (int)floor(f4 * G + 0.5);
  std::vector<float> W((size_t)N * K);
  std::normal_distribution<float> nd(0.f, 0.02f);
  for (auto& w : W) w = nd(rng);
  const mpq_desc d = {N, K, g1, g2, axis};
  int64_t cap = 0;
  CHECK(mpq_quantize_outlier_capacity(&d, n4, p_o, &cap) == MPQ_OK);
  const int S2 = axis == 0 ? N * ((G + g2 - 1) / g2) : ((N + g2 - 1) / g2) * G;
  std::vector<uint8_t> is4(G), codes((size_t)N * K), s_int((size_t)N * G), z1((size_t)N * G);
  std::vector<uint16_t> s2(S2), z2(S2), col(cap + 1), val(cap + 1);
  std::vector<int32_t> row_ptr(N + 1);
  mpq_logical_out out = {is4.data(), codes.data(), s_int.data(), z1.data(), s2.data(), z2.data(), row_ptr.data(), col.data(), val.data()};
  int64_t nnz = -1;
  CHECK(mpq_quantize_host(&d, W.data(), n4, p_o, &out, cap, &nnz) == MPQ_OK);
  CHECK(nnz >= 0 && nnz <= cap && row_ptr[N] == nnz);
  CHECK(mpq_quantize_host(&d, W.data(), n4, p_o, &out, cap > 0 ? cap - 1 : -1, &nnz) != MPQ_OK);  // too small / invalid capacity
  const mpq_logical lg = {is4.data(), codes.data(), s_int.data(), z1.data(), s2.data(), z2.data(), row_ptr.data(), col.data(), val.data()};
  size_t bytes = 0;
  CHECK(mpq_packed_size(&d, is4.data(), row_ptr.data(), &bytes) == MPQ_OK && bytes >= MPQ_HEADER_BYTES);
  std::vector<uint8_t> blob(bytes);
  CHECK(mpq_pack_host(&d, &lg, blob.data(), bytes - 1) == MPQ_ERR_SIZE);
  CHECK(mpq_pack_host(&d, &lg, blob.data(), bytes) == MPQ_OK);
  mpq_desc back;
  int64_t nnz_b = 0;
  int32_t n4_b = 0;
  uint64_t total = 0;
  CHECK(mpq_blob_info(blob.data(), &back, &nnz_b, &n4_b, &total) == MPQ_OK);
  CHECK(back.N == N && back.K == K && nnz_b == nnz && n4_b == n4 && total == bytes);
  uint64_t first = 0, rec = 0;
  int32_t cnt = 0;
  CHECK(mpq_blob_tiles(blob.data(), &first, &rec, &cnt) == MPQ_OK && cnt == (N + 15) / 16 && first + rec * cnt <= bytes);
  blob[9] ^= 0x40;  // a header that is not what the packer writes
  CHECK(mpq_blob_tiles(blob.data(), &first, &rec, &cnt) == MPQ_ERR_BLOB);
  // malformed inputs
  if (nnz > 0 && n4 > 0) {
    std::vector<uint16_t> col2(col);
    int g4 = 0;
    while (!is4[g4]) ++g4;
    col2[0] = (uint16_t)(g4 * g1);
    const mpq_logical bad = {is4.data(), codes.data(), s_int.data(), z1.data(), s2.data(), z2.data(), row_ptr.data(), col2.data(), val.data()};
    const mpq_status st = mpq_pack_host(&d, &bad, blob.data(), bytes);
    CHECK(st == MPQ_ERR_OUTLIER_IN_4BIT || st == MPQ_ERR_CSR);
  }
  {
    std::vector<uint8_t> codes2(codes);
    int g2bit = 0;
    while (g2bit < G && is4[g2bit]) ++g2bit;
    if (g2bit < G) {
      codes2[(size_t)g2bit * g1] = 4;
      const mpq_logical bad = {is4.data(), codes2.data(), s_int.data(), z1.data(), s2.data(), z2.data(), row_ptr.data(), col.data(), val.data()};
      CHECK(mpq_pack_host(&d, &bad, blob.data(), bytes) == MPQ_ERR_CODE_RANGE);
    }
  }
  // the oracle on the same logical matrix
  const orc_desc od = {N, K, g1, g2, axis};
  CHECK(orc_validate(&od, is4.data(), codes.data(), row_ptr.data(), col.data()) == 0);
  std::vector<uint16_t> Wd((size_t)N * K);
  orc_dequant(&od, codes.data(), s_int.data(), z1.data(), s2.data(), z2.data(), row_ptr.data(), col.data(), val.data(), 1, Wd.data());
  const int M = 3;
  std::vector<uint16_t> X((size_t)M * K);
  for (auto& x : X) x = orc_float_to_half(nd(rng) * 50.f);
  std::vector<double> Y((size_t)M * N, NAN);
  orc_gemm_rows(&od, codes.data(), s_int.data(), z1.data(), s2.data(), z2.data(), row_ptr.data(), col.data(), val.data(), X.data(), M, 0, N, 2, Y.data());
  for (double y : Y) CHECK(isfinite(y));
  const double stored = orc_avg_bits_stored(&od, n4, nnz), lib = mpq_avg_bits(&d, n4, nnz, 0, 4);
  CHECK(fabs(stored - lib) < 1e-9);
  return 0;
}

int main() {
  int rc = 0;
  rc |= one(40, 512, 64, 16, 0, 0.10, 0.005, 1);
  rc |= one(37, 704, 64, 4, 0, 0.30, 0.02, 2);      // ragged rows, short last super-group
  rc |= one(20, 1024, 128, 2, 0, 0.25, 0.01, 3);
  rc |= one(40, 512, 16, 16, 1, 0.25, 0.01, 4);     // the paper's operating point
  rc |= one(70, 480, 32, 32, 1, 0.20, 0.01, 5);
  rc |= one(16, 512, 64, 16, 0, 1.0, 0.0, 6);       // only 4-bit groups
  rc |= one(5, 64, 64, 1, 0, 0.0, 0.2, 7);          // a single group
  mpq_desc bad = {8, 100, 64, 16, 0};
  size_t bytes = 0;
  uint8_t is4[2] = {0, 0};
  int32_t rp[9] = {0};
  if (mpq_packed_size(&bad, is4, rp, &bytes) != MPQ_ERR_SHAPE) { fprintf(stderr, "K %% g1 != 0 accepted\n"); rc = 1; }
  if (mpq_avg_bits(nullptr, 0, 0, 0, 4) >= 0) { fprintf(stderr, "null desc accepted\n"); rc = 1; }
  printf(rc ? "FAILED\n" : "ok\n");
  return rc;
}
