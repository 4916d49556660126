// mpq_kernels.hip - gfx950 kernels and device entry points of the mixed-precision weight library.
//
// Kernels (all read the packed blob described in mpq_format.h):
//   mpq_gemv_kernel     Algorithm 1 (GEMV with asynchronous dequantization) re-designed for CDNA4,
//                       with the outlier product of Sec. 4.3 fused in as a per-row correction.
//   mpq_dequant_kernel  eq. 5 applied twice (scale, then weight), written out as row-major fp16.
//   mpq_outlier_add_kernel  adds the CSR values to a dequantized matrix (dense + sparse, Sec. 2.3).
//
// Mapping shared by the kernels.  A workgroup owns one tile of 16 rows for all of K.  A wavefront
// load of 1 KiB is one block: lane = j*16 + i holds the 16-byte unit j (of 4) of row i (of 16).
// The waves of the workgroup take the tile's blocks round-robin, first the 2-bit stream, then the
// 4-bit stream.  A lane therefore always decodes codes of ONE row and ONE first-order group, so
// the group's scale and zero point are per-lane scalars.
//
// Per-weight arithmetic (bit-exact to the definition in mpq.h):
//   a mask isolates two codes (low / high half-word of a dword); OR-ing 0x6400 into each half
//   makes the fp16 numbers 1024 + c*4^p; one packed fma (x 4^-p, - (1024*4^-p + z1)) gives the
//   exact integers c - z1; one packed fp16 multiply by s1 is the rounding the definition asks
//   for.  The GEMV then feeds the pair to v_dot2_f32_f16 (fp32 accumulation).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mpq.h"
#include "mpq_format.h"

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

#define XS_STRIDE 144 /* LDS bytes per 64 activations: 128 B + 16 B skew against bank conflicts */

struct DevBlob {
  const uint32_t* unit2;
  const uint32_t* unit4;
  const uint4* codes2;
  const uint4* codes4;
  const uint16_t* meta1;
  const uint32_t* meta2;
  const int32_t* rowptr;
  const uint32_t* outl;
  int32_t N, K, G, S, n2, U2, U4, B2, B4, T;
};

__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t as_u32(half2_t h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ half_t bits_to_half(uint16_t u) { return __builtin_bit_cast(half_t, u); }
__device__ __forceinline__ uint16_t half_to_bits(half_t h) { return __builtin_bit_cast(uint16_t, h); }

// Waits for this wave's LDS traffic only, then meets the other waves.  Global loads that are still
// in flight (prefetched code blocks) stay in flight, which __syncthreads() would not allow.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Second-order dequantization of a first-order scale: fp16((fp32(s_int) - fp32(z2)) * fp32(s2)).
// (Algorithm 1, "1st s <- dequantize(1st s_int, 2nd z, 2nd s)"; eq. 5 form.)
__device__ __forceinline__ half_t scale_dequant(uint32_t s_int, uint32_t m2) {
#pragma clang fp contract(off)
  const float z2 = (float)bits_to_half((uint16_t)(m2 >> 16));
  const float s2 = (float)bits_to_half((uint16_t)(m2 & 0xFFFFu));
  const float t = (float)s_int - z2;
  float u = t * s2;
  // The product must be rounded to binary32 before it is rounded to fp16 (two roundings, as the
  // definition states).  Without this barrier the compiler folds multiply and conversion into
  // v_fma_mixlo_f16, which rounds once and differs in the last bit for about one scale in 10^4.
  asm volatile("" : "+v"(u));
  return (half_t)u;
}

// First-order dequantization (eq. 5) of one 2-bit unit: 64 codes -> 32 fp16 pairs, pair r holding
// columns (2r, 2r+1) of the unit.
__device__ __forceinline__ void decode2(const uint4 q, const half_t s1, const half_t z1h, half2_t (&w)[32]) {
#pragma clang fp contract(off)
  const uint32_t magic = 0x64006400u;  // fp16 1024.0 in both halves
  const half2_t s1p = {s1, s1};
  half2_t nb[5], sc[5];
  const float inv[5] = {1.0f, 0.25f, 0.0625f, 0.015625f, 0.00390625f};
#pragma unroll
  for (int p = 0; p < 5; ++p) {
    const half_t b = (half_t)(-1024.0f * inv[p]) - z1h;  // exact: integer below 2048
    nb[p] = half2_t{b, b};
    sc[p] = half2_t{(half_t)inv[p], (half_t)inv[p]};
  }
  const uint32_t qd[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t lo = qd[d];
    const uint32_t hi = qd[d] >> 10;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int pp = p < 5 ? p : p - 5;
      const uint32_t src = p < 5 ? lo : hi;
      const half2_t h = as_h2((src & (0x00030003u << (2 * pp))) | magic);
      const half2_t dz = __builtin_elementwise_fma(h, sc[pp], nb[pp]);  // exact c - z1
      w[4 * p + d] = dz * s1p;
    }
  }
}

// The same for one 4-bit unit: 32 codes -> 16 pairs.
__device__ __forceinline__ void decode4(const uint4 q, const half_t s1, const half_t z1h, half2_t (&w)[16]) {
#pragma clang fp contract(off)
  const uint32_t magic = 0x64006400u;
  const half2_t s1p = {s1, s1};
  const half_t b0 = (half_t)(-1024.0f) - z1h, b1 = (half_t)(-64.0f) - z1h;
  const half2_t nb[2] = {half2_t{b0, b0}, half2_t{b1, b1}};
  const half2_t sc[2] = {half2_t{(half_t)1.0f, (half_t)1.0f}, half2_t{(half_t)0.0625f, (half_t)0.0625f}};
  const uint32_t qd[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t lo = qd[d];
    const uint32_t hi = qd[d] >> 8;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int pp = p & 1;
      const uint32_t src = p < 2 ? lo : hi;
      const half2_t h = as_h2((src & (0x000F000Fu << (4 * pp))) | magic);
      const half2_t dz = __builtin_elementwise_fma(h, sc[pp], nb[pp]);
      w[4 * p + d] = dz * s1p;
    }
  }
}

__device__ __forceinline__ float dot2(half2_t a, uint32_t xb, float acc) {
  return __builtin_amdgcn_fdot2(a, as_h2(xb), acc, false);
}

// Description of what one lane has to do for block c of the current tile.
struct LaneBlock {
  uint4 q;
  uint32_t m1;
};

template <int G1>
__device__ __forceinline__ void issue_block(const DevBlob& b, int tile, int c, int lane, LaneBlock& out) {
  const int i = lane & 15, j = lane >> 4;
  const uint16_t* m1t = b.meta1 + (size_t)tile * b.G * 16 + i;
  if (c < b.B2) {
    out.q = b.codes2[((size_t)tile * b.B2 + c) * 64 + lane];
    const int u = 4 * c + j;
    const int sg = G1 == 64 ? u : (u >> 1);
    out.m1 = u < b.U2 ? (uint32_t)m1t[sg * 16] : 0u;
  } else {
    const int c4 = c - b.B2;
    out.q = b.codes4[((size_t)tile * b.B4 + c4) * 64 + lane];
    const int u = 4 * c4 + j;
    const int sg = b.n2 + (G1 == 64 ? (u >> 1) : (u >> 2));
    out.m1 = u < b.U4 ? (uint32_t)m1t[sg * 16] : 0u;
  }
}

// ------------------------------------------------------------------------------------ GEMV
//
// LDS: activations (skewed), unit tables of both streams, the tile's second-order pairs, and the
// cross-wave reduction slots.
template <int G1>
__global__ void __launch_bounds__(1024)
mpq_gemv_kernel(const DevBlob b, const uint16_t* __restrict__ x, uint16_t* __restrict__ y) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int lane = tid & 63, wv = tid >> 6, W = nthr >> 6;
  const int i = lane & 15, j = lane >> 4;
  const int C = b.B2 + b.B4;
  unsigned char* xs = smem;
  const int xs_bytes = (b.K >> 6) * XS_STRIDE;
  uint32_t* units = (uint32_t*)(smem + xs_bytes);
  uint32_t* m2s = units + 4 * C;
  float* red = (float*)(m2s + b.S * 16);
  float* ored = red + W * 16;

  // threads-per-row mapping of the outlier phase: 16 rows share the workgroup's threads
  const int tpr = nthr >> 4;
  const int orow = tid / tpr, oq = tid % tpr;

  bool staged = false;
  for (int tile = blockIdx.x; tile < b.T; tile += gridDim.x) {
    // (1) everything this tile needs from global memory is requested up front: row pointers, the
    //     first code block of this wave, then the small operands that go to LDS.
    const int32_t rp0 = b.rowptr[tile * 16 + orow];
    const int32_t rp1 = b.rowptr[tile * 16 + orow + 1];
    LaneBlock cur, nxt;
    int c = wv;
    if (c < C) issue_block<G1>(b, tile, c, lane, cur);
    if (c + W < C) issue_block<G1>(b, tile, c + W, lane, nxt);
    if (!staged) {
      for (int ch = tid; ch < (b.K >> 3); ch += nthr) {
        const uint4 v = ((const uint4*)x)[ch];
        const int k = ch << 3;
        *(uint4*)(xs + (k >> 6) * XS_STRIDE + (k & 63) * 2) = v;
      }
      for (int u = tid; u < 4 * b.B2; u += nthr) units[u] = b.unit2[u];
      for (int u = tid; u < 4 * b.B4; u += nthr) units[4 * b.B2 + u] = b.unit4[u];
      staged = true;
    }
    for (int e = tid; e < b.S * 16; e += nthr) m2s[e] = b.meta2[(size_t)tile * b.S * 16 + e];
    lds_barrier();

    // (2) first outlier words of this thread's row (the rest are fetched in the tail loop)
    uint32_t o0 = 0, o1 = 0;
    const int32_t e0 = rp0 + oq, e1 = e0 + tpr;
    if (e0 < rp1) o0 = b.outl[e0];
    if (e1 < rp1) o1 = b.outl[e1];

    // (3) main loop over this wave's blocks: the next block's loads are in flight while the
    //     current block's scale is reconstructed and its codes are decoded and multiplied.
    float acc0 = 0.f, acc1 = 0.f;
    for (; c < C; c += W) {
      const LaneBlock blk = cur;
      cur = nxt;
      if (c + 2 * W < C) issue_block<G1>(b, tile, c + 2 * W, lane, nxt);
      const uint32_t ue = units[4 * c + j];
      const bool valid = ue != MPQ_INVALID_UNIT;
      const uint32_t k0 = valid ? (ue & 0xFFFFu) * 32u : 0u;
      const uint32_t sgp = valid ? (ue >> 16) : 0u;
      const uint32_t m2 = m2s[sgp * 16 + i];
      half_t s1 = scale_dequant(blk.m1 & 0xFFu, m2);
      if (!valid) s1 = (half_t)0.0f;
      const half_t z1h = (half_t)(float)(blk.m1 >> 8);
      const unsigned char* xu = xs + (k0 >> 6) * XS_STRIDE + (k0 & 63u) * 2u;
      if (c < b.B2) {
        half2_t w[32];
        decode2(blk.q, s1, z1h, w);
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const uint4 xv = *(const uint4*)(xu + 16 * p);
          acc0 = dot2(w[4 * p + 0], xv.x, acc0);
          acc1 = dot2(w[4 * p + 1], xv.y, acc1);
          acc0 = dot2(w[4 * p + 2], xv.z, acc0);
          acc1 = dot2(w[4 * p + 3], xv.w, acc1);
        }
      } else {
        half2_t w[16];
        decode4(blk.q, s1, z1h, w);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const uint4 xv = *(const uint4*)(xu + 16 * p);
          acc0 = dot2(w[4 * p + 0], xv.x, acc0);
          acc1 = dot2(w[4 * p + 1], xv.y, acc1);
          acc0 = dot2(w[4 * p + 2], xv.z, acc0);
          acc1 = dot2(w[4 * p + 3], xv.w, acc1);
        }
      }
    }
    float acc = acc0 + acc1;
    // (4) the four unit columns of a row sit in lanes i, i+16, i+32, i+48
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (lane < 16) red[wv * 16 + lane] = acc;

    // (5) outliers of row `orow`: sum val * x[col] over the row's CSR words (Sec. 4.3, fused)
    float oacc = 0.f;
    {
      auto use = [&](uint32_t word) {
        const uint32_t col = word & 0xFFFFu;
        const half_t xv = *(const half_t*)(xs + (col >> 6) * XS_STRIDE + (col & 63u) * 2u);
        oacc += (float)bits_to_half((uint16_t)(word >> 16)) * (float)xv;
      };
      if (e0 < rp1) use(o0);
      if (e1 < rp1) use(o1);
      for (int32_t e = e1 + tpr; e < rp1; e += tpr) use(b.outl[e]);
      for (int off = tpr >> 1; off > 0; off >>= 1) oacc += __shfl_xor(oacc, off);
      if (oq == 0) ored[orow] = oacc;
    }
    lds_barrier();
    if (tid < 16) {
      float tot = ored[tid];
      for (int w2 = 0; w2 < W; ++w2) tot += red[w2 * 16 + tid];
      const int row = tile * 16 + tid;
      if (row < b.N) y[row] = half_to_bits((half_t)tot);
    }
    if (tile + (int)gridDim.x < b.T) lds_barrier();  // red / m2s are rewritten by the next tile
  }
}

// ------------------------------------------------------------------------------------ dequant
template <int G1>
__global__ void __launch_bounds__(256)
mpq_dequant_kernel(const DevBlob b, uint16_t* __restrict__ Wout) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6, W = blockDim.x >> 6;
  const int i = lane & 15, j = lane >> 4;
  const int C = b.B2 + b.B4;
  const int tile = blockIdx.x;
  const int row = tile * 16 + i;
  for (int c = wv; c < C; c += W) {
    LaneBlock blk;
    issue_block<G1>(b, tile, c, lane, blk);
    const uint32_t ue = c < b.B2 ? b.unit2[4 * c + j] : b.unit4[4 * (c - b.B2) + j];
    if (ue == MPQ_INVALID_UNIT || row >= b.N) continue;
    const uint32_t k0 = (ue & 0xFFFFu) * 32u;
    const uint32_t m2 = b.meta2[((size_t)tile * b.S + (ue >> 16)) * 16 + i];
    const half_t s1 = scale_dequant(blk.m1 & 0xFFu, m2);
    const half_t z1h = (half_t)(float)(blk.m1 >> 8);
    uint4* dst = (uint4*)(Wout + (size_t)row * b.K + k0);
    if (c < b.B2) {
      half2_t w[32];
      decode2(blk.q, s1, z1h, w);
#pragma unroll
      for (int p = 0; p < 8; ++p)
        dst[p] = uint4{as_u32(w[4 * p]), as_u32(w[4 * p + 1]), as_u32(w[4 * p + 2]), as_u32(w[4 * p + 3])};
    } else {
      half2_t w[16];
      decode4(blk.q, s1, z1h, w);
#pragma unroll
      for (int p = 0; p < 4; ++p)
        dst[p] = uint4{as_u32(w[4 * p]), as_u32(w[4 * p + 1]), as_u32(w[4 * p + 2]), as_u32(w[4 * p + 3])};
    }
  }
}

// One thread per (row, slot): W[row][col] = fp16(W[row][col] + val)  (native fp16 add = the fp32
// add followed by one rounding that the definition states).
__global__ void __launch_bounds__(256)
mpq_outlier_add_kernel(const DevBlob b, uint16_t* __restrict__ Wout) {
  const int tpr = blockDim.x >> 4;
  const int row = blockIdx.x * 16 + threadIdx.x / tpr;
  const int oq = threadIdx.x % tpr;
  if (row >= b.N) return;
  const int32_t rp0 = b.rowptr[row], rp1 = b.rowptr[row + 1];
  for (int32_t e = rp0 + oq; e < rp1; e += tpr) {
    const uint32_t word = b.outl[e];
    uint16_t* at = Wout + (size_t)row * b.K + (word & 0xFFFFu);
    const half_t s = bits_to_half(*at) + bits_to_half((uint16_t)(word >> 16));
    *at = half_to_bits(s);
  }
}

// ------------------------------------------------------------------------------------ host side

namespace {

mpq_status make_dev(const void* hdr_host, const void* blob_dev, MpqHeader* h, DevBlob* d) {
  if (!hdr_host || !blob_dev) return MPQ_ERR_NULL;
  mpq_status st = mpq_internal_check_header(hdr_host, h);
  if (st != MPQ_OK) return st;
  if (((uintptr_t)blob_dev & 15u) != 0) return MPQ_ERR_ALIGN;
  const unsigned char* p = (const unsigned char*)blob_dev;
  d->unit2 = (const uint32_t*)(p + h->off_unit2);
  d->unit4 = (const uint32_t*)(p + h->off_unit4);
  d->codes2 = (const uint4*)(p + h->off_codes2);
  d->codes4 = (const uint4*)(p + h->off_codes4);
  d->meta1 = (const uint16_t*)(p + h->off_meta1);
  d->meta2 = (const uint32_t*)(p + h->off_meta2);
  d->rowptr = (const int32_t*)(p + h->off_rowptr);
  d->outl = (const uint32_t*)(p + h->off_outl);
  d->N = h->N; d->K = h->K; d->G = h->G; d->S = h->S; d->n2 = h->n2;
  d->U2 = h->U2; d->U4 = h->U4; d->B2 = h->B2; d->B4 = h->B4; d->T = h->T;
  return MPQ_OK;
}

int g_gemv_threads = 0;  // 0 = choose from K
int g_gemv_max_blocks = 0;

size_t gemv_lds_bytes(const MpqHeader& h, int threads) {
  const size_t W = threads / 64;
  return (size_t)(h.K / 64) * XS_STRIDE + 16ull * (h.B2 + h.B4) + 64ull * h.S + (W * 16 + 16) * 4;
}

template <typename Kern>
mpq_status allow_lds(Kern kern, size_t bytes) {
  if (bytes > 160 * 1024) return MPQ_ERR_UNSUPPORTED;
  if (bytes > 48 * 1024) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
      (void)hipGetLastError();
      return MPQ_ERR_HIP;
    }
  }
  return MPQ_OK;
}

}  // namespace

extern "C" {

// Launch-shape override for tuning sweeps (0 restores the built-in choice). Not thread safe.
void mpq_debug_set_gemv_launch(int threads, int max_blocks) {
  g_gemv_threads = threads;
  g_gemv_max_blocks = max_blocks;
}

mpq_status mpq_gemv(const void* hdr_host, const void* blob_dev, const uint16_t* x_dev, uint16_t* y_dev,
                    void* stream) {
  if (!x_dev || !y_dev) return MPQ_ERR_NULL;
  MpqHeader h;
  DevBlob d;
  mpq_status st = make_dev(hdr_host, blob_dev, &h, &d);
  if (st != MPQ_OK) return st;
  if ((((uintptr_t)x_dev | (uintptr_t)y_dev) & 15u) != 0) return MPQ_ERR_ALIGN;
  int threads = g_gemv_threads > 0 ? g_gemv_threads : (h.K > 16384 ? 512 : 256);
  if (threads % 64 != 0 || threads < 64 || threads > 1024) return MPQ_ERR_SHAPE;
  const size_t lds = gemv_lds_bytes(h, threads);
  int blocks = h.T;
  if (g_gemv_max_blocks > 0 && blocks > g_gemv_max_blocks) blocks = g_gemv_max_blocks;
  hipStream_t s = (hipStream_t)stream;
  if (h.g1 == 64) {
    st = allow_lds(mpq_gemv_kernel<64>, lds);
    if (st != MPQ_OK) return st;
    hipLaunchKernelGGL(mpq_gemv_kernel<64>, dim3(blocks), dim3(threads), lds, s, d, x_dev, y_dev);
  } else {
    st = allow_lds(mpq_gemv_kernel<128>, lds);
    if (st != MPQ_OK) return st;
    hipLaunchKernelGGL(mpq_gemv_kernel<128>, dim3(blocks), dim3(threads), lds, s, d, x_dev, y_dev);
  }
  return hipGetLastError() == hipSuccess ? MPQ_OK : MPQ_ERR_HIP;
}

mpq_status mpq_dequant(const void* hdr_host, const void* blob_dev, uint16_t* W_out_dev, int add_outliers,
                       void* stream) {
  if (!W_out_dev) return MPQ_ERR_NULL;
  MpqHeader h;
  DevBlob d;
  mpq_status st = make_dev(hdr_host, blob_dev, &h, &d);
  if (st != MPQ_OK) return st;
  if (((uintptr_t)W_out_dev & 15u) != 0) return MPQ_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  if (h.g1 == 64)
    hipLaunchKernelGGL(mpq_dequant_kernel<64>, dim3(h.T), dim3(256), 0, s, d, W_out_dev);
  else
    hipLaunchKernelGGL(mpq_dequant_kernel<128>, dim3(h.T), dim3(256), 0, s, d, W_out_dev);
  if (hipGetLastError() != hipSuccess) return MPQ_ERR_HIP;
  if (add_outliers && h.nnz > 0) {
    hipLaunchKernelGGL(mpq_outlier_add_kernel, dim3(h.T), dim3(256), 0, s, d, W_out_dev);
    if (hipGetLastError() != hipSuccess) return MPQ_ERR_HIP;
  }
  return MPQ_OK;
}

}  // extern "C"

extern "C" mpq_status mpq_gemm(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev,
                               uint16_t* Y_dev, int32_t M, void* stream) {
  if (!X_dev || !Y_dev) return MPQ_ERR_NULL;
  if (M < 1 || M > MPQ_MAX_M) return MPQ_ERR_SHAPE;
  MpqHeader h;
  mpq_status st = mpq_internal_check_header(hdr_host, &h);
  if (st != MPQ_OK) return st;
  // Row m of the batch is an independent matrix-vector product.
  for (int32_t m = 0; m < M; ++m) {
    st = mpq_gemv(hdr_host, blob_dev, X_dev + (size_t)m * h.K, Y_dev + (size_t)m * h.N, stream);
    if (st != MPQ_OK) return st;
  }
  return MPQ_OK;
}
