// mpq_kernels.hip - gfx950 kernels and device entry points of the mixed-precision weight library.
//
// Kernels (all read the packed blob described in mpq_format.h):
//   mpq_mm_kernel        Algorithm 1 (GEMV with asynchronous dequantization) re-designed for CDNA4,
//                        for a batch of 1..32 activation rows, with the outlier product of
//                        Sec. 4.3 fused in as a per-row correction.
//   mpq_dequant_kernel   eq. 5 applied twice (scale, then weight), written out as row-major fp16.
//   mpq_outlier_add_kernel  adds the CSR values to a dequantized matrix (dense + sparse, Sec. 2.3).
//
// Mapping shared by the kernels.  A workgroup owns one tile of 16 rows for all of K.  A wavefront
// load of 1 KiB is one block: lane = j*16 + i holds the 16-byte unit j (of 4) of row i (of 16).
// The four waves of the workgroup take the tile's blocks round-robin, first the 2-bit stream,
// then the 4-bit stream.  A lane therefore always decodes codes of ONE row and ONE first-order
// group, so the group's scale and zero point are per-lane scalars.
//
// Per-weight arithmetic (bit-exact to the definition in mpq.h):
//   a mask isolates two codes (low / high half-word of a dword); OR-ing 0x6400 into each half
//   makes the fp16 numbers 1024 + c*4^p; one packed fma (x 4^-p, - (1024*4^-p + z1)) gives the
//   exact integers c - z1; one packed fp16 multiply by s1 is the rounding the definition asks
//   for.  The product kernel hands the resulting pairs to the matrix core.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mpq.h"
#include "mpq_format.h"

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;

struct DevBlob {
  const uint2* unit2;
  const uint2* unit4;
  const uint4* codes2;
  const uint4* codes4;
  const uint16_t* meta1;
  const uint32_t* meta2;
  const unsigned char* otile;  // per-tile outlier records
  int32_t N, K, G, S, n2, U2, U4, B2, B4, T;
  int32_t orec_bytes;          // bytes of one outlier record (row-start table + words), 0 if no outliers
  int64_t nnz;
  int32_t dbg;  // tuning experiments only: bit 0 skips the decode/multiply, bit 1 skips the code-block loads
};

__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t as_u32(half2_t h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ half_t bits_to_half(uint16_t u) { return __builtin_bit_cast(half_t, u); }
__device__ __forceinline__ uint16_t half_to_bits(half_t h) { return __builtin_bit_cast(uint16_t, h); }

// Waits for this wave's LDS traffic only, then meets the other waves.  Global loads that are still
// in flight (code blocks on their way to LDS) stay in flight, which __syncthreads() would not allow.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// s_waitcnt vmcnt(n) for a wave-uniform n known only at run time (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "do not wait").  Larger n wait for vmcnt(9),
// which is stricter and therefore safe.
#define MPQ_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
__device__ __forceinline__ void wait_vm(int n) {
  switch (n) {
    case 0: MPQ_VMCNT(0); break;
    case 1: MPQ_VMCNT(1); break;
    case 2: MPQ_VMCNT(2); break;
    case 3: MPQ_VMCNT(3); break;
    case 4: MPQ_VMCNT(4); break;
    case 5: MPQ_VMCNT(5); break;
    case 6: MPQ_VMCNT(6); break;
    case 7: MPQ_VMCNT(7); break;
    case 8: MPQ_VMCNT(8); break;
    default: MPQ_VMCNT(9); break;
  }
}

// The product kernel issues its global loads with inline asm and waits for them with explicit
// s_waitcnt vmcnt(n): the compiler's own wait insertion cannot count requests issued in loops and
// would otherwise wait for ALL outstanding loads (vmcnt(0)) whenever LDS written by a direct load
// is read, which serialises the whole pipeline.  Values loaded this way must not be used before
// the matching wait_vm().

// 16 bytes per lane straight from global memory into LDS at lds + 16*lane (no register staging).
__device__ __forceinline__ void dma16(const void* g, unsigned char* lds_wave_uniform) {
  const uint32_t l = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_wave_uniform);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(l), "v"(g) : "memory");
}

// One dword per lane into a register, asynchronously.
__device__ __forceinline__ uint32_t load_b32_async(const void* g) {
  uint32_t r;
  asm volatile("global_load_dword %0, %1, off" : "=v"(r) : "v"(g) : "memory");
  return r;
}

// Copies `bytes` (a multiple of 16) to LDS with the waves of a 256-thread workgroup taking 1 KiB
// pieces in turn.
__device__ __forceinline__ void dma_region(const void* g, unsigned char* l, int bytes, int wv, int lane) {
  for (int ch = wv; ch * 1024 < bytes; ch += 4) {
    const int off = ch * 1024 + lane * 16;
    if (off < bytes) dma16((const unsigned char*)g + off, l + ch * 1024);
  }
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

// Constants of the decode kept in scalar registers so that v_and_or_b32 / v_pk_fma_f16 can take
// them as operands (VOP3 encodings on gfx9 have no literal operands).
__device__ __forceinline__ uint32_t sgpr_const(uint32_t v) {
  uint32_t r;
  asm volatile("s_mov_b32 %0, %1" : "=s"(r) : "i"(v));
  return r;
}

struct DecodeConsts {
  uint32_t mask2[5], mask4[2], sc2[5], sc4[2];
  uint32_t magic;
};

__device__ __forceinline__ DecodeConsts make_consts() {
  DecodeConsts k;
  k.mask2[0] = sgpr_const(0x00030003u); k.mask2[1] = sgpr_const(0x000C000Cu); k.mask2[2] = sgpr_const(0x00300030u);
  k.mask2[3] = sgpr_const(0x00C000C0u); k.mask2[4] = sgpr_const(0x03000300u);
  k.mask4[0] = sgpr_const(0x000F000Fu); k.mask4[1] = sgpr_const(0x00F000F0u);
  k.sc2[0] = sgpr_const(0x3C003C00u);  // 1
  k.sc2[1] = sgpr_const(0x34003400u);  // 1/4
  k.sc2[2] = sgpr_const(0x2C002C00u);  // 1/16
  k.sc2[3] = sgpr_const(0x24002400u);  // 1/64
  k.sc2[4] = sgpr_const(0x1C001C00u);  // 1/256
  k.sc4[0] = k.sc2[0];
  k.sc4[1] = k.sc2[2];
  asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(k.magic));  // fp16 1024.0 in both halves
  return k;
}

// First-order dequantization (eq. 5) of step P of a unit: the four dwords give the four fp16 pairs
// of columns 8P .. 8P+7.  TWO_BIT selects 2-bit (P = 0..7) or 4-bit (P = 0..3) fields.
// zb = fp16(1024 + z1); lo / hi = the unit's dwords and the same shifted right by 10 (2-bit) or 8
// (4-bit) so that every field sits in mantissa bits.
template <bool TWO_BIT, int P>
__device__ __forceinline__ uint4 decode_step(const uint32_t (&lo)[4], const uint32_t (&hi)[4], const half2_t s1p,
                                             const half_t zb, const DecodeConsts& kc) {
#pragma clang fp contract(off)
  constexpr int pp = TWO_BIT ? (P < 5 ? P : P - 5) : (P & 1);
  constexpr bool shifted = TWO_BIT ? (P >= 5) : (P >= 2);
  // -(1024 * f + z1) with f = 4^-pp (2-bit) or 16^-pp (4-bit): exact, an integer below 2048
  constexpr float off = TWO_BIT ? (pp == 0 ? 0.f : pp == 1 ? 768.f : pp == 2 ? 960.f : pp == 3 ? 1008.f : 1020.f)
                                : (pp == 0 ? 0.f : 960.f);
  const half_t t = (half_t)off - zb;
  const half2_t nb = {t, t};
  const uint32_t mask = TWO_BIT ? kc.mask2[pp] : kc.mask4[pp];
  const half2_t sc = as_h2(TWO_BIT ? kc.sc2[pp] : kc.sc4[pp]);
  uint32_t a[4];
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t src = shifted ? hi[d] : lo[d];
    const half2_t h = as_h2((src & mask) | kc.magic);           // 1024 + c / f
    const half2_t dz = __builtin_elementwise_fma(h, sc, nb);    // exact c - z1
    a[d] = as_u32(dz * s1p);                                    // fp16((c - z1) * s1)
  }
  return uint4{a[0], a[1], a[2], a[3]};
}

// ------------------------------------------------------------------------------------ product
//
// Y[m][n] = sum_k X[m][k] W[n][k] + outliers, 1 <= M <= 16*NT, one 16-row tile per workgroup.
//
// Data movement (the "asynchronous dequantization" of Sec. 5 on this hardware): everything the
// tile needs is requested in the first instructions of the workgroup and lands in LDS without
// passing through registers (global_load_lds_dwordx4): the activations, the unit tables, the
// tile's (s_int, z1) and (s2, z2) words, the tile's outlier record, and PD code blocks per wave.  While the code blocks are
// still in flight the waves meet once, and then every wave consumes its blocks in order, waiting
// with s_waitcnt vmcnt(n) only for the block it needs next and refilling the freed slot.  The
// second-order scale reconstruction of a block runs while the later blocks are still on their way.
//
// Compute: the decoded fp16 weights of a block are exactly the A operand of
// v_mfma_f32_16x16x32_f16 (lane j*16+i holds 8 consecutive columns of row i), the activations of
// the same columns are the B operand (lane j*16+m holds X[m][same 8 columns]), and the 16x16 fp32
// accumulator holds Y[m][row] for the whole tile.  The matrix core does the multiply-accumulate
// and the reduction over the four unit columns, so the vector ALU only decodes.  Batch columns
// beyond M compute garbage that is never stored.
//
// LDS: `ring` (PD slots of 1 KiB per wave, reused for the cross-wave reduction at the end) and
// `stage` are separate objects so that the compiler can tell reads of `stage` from the direct
// loads into `ring`; ring slots are read with inline asm after an explicit wait.
template <int NT, int PD, int STB>
__global__ void __launch_bounds__(256)
mpq_mm_kernel(const DevBlob b, const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, const int M) {
#pragma clang fp contract(off)
  static_assert(PD >= NT && PD <= 8, "ring depth");
  __shared__ __align__(16) unsigned char ring[4 * PD * 1024];
  __shared__ __align__(16) unsigned char stage[STB];
  constexpr int W = 4;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, j = lane >> 4;
  const int C = b.B2 + b.B4;
  const int tile = blockIdx.x;
  // stage layout: unit tables | meta1 of the tile | meta2 of the tile | outlier record | activation rows
  const int units_bytes = 32 * C, m1_bytes = 32 * b.G, m2_bytes = 64 * b.S;
  const int rowbytes = 2 * b.K + 16;  // + 16: rows of a batch start in different LDS banks
  unsigned char* units = stage;
  unsigned char* m1s = units + units_bytes;
  unsigned char* m2s = m1s + m1_bytes;
  unsigned char* ots = m2s + m2_bytes;
  unsigned char* xs = ots + b.orec_bytes;
  unsigned char* myring = ring + wv * (PD * 1024);
  const DecodeConsts kc = make_consts();

  // outlier / output mapping: 16 consecutive lanes share a row; lane q handles batch column q % Mp
  // and every (16/Mp)-th outlier of the row
  const int orow = tid >> 4, oq = tid & 15;
  int Mp = 1;
  while (Mp < M && Mp < 16) Mp <<= 1;
  const int om = oq & (Mp - 1), oes = oq / Mp, ostride = 16 / Mp;

  // ---- (1) all requests of the tile, oldest first: staged operands, then code blocks
  dma_region(b.unit2, units, 32 * b.B2, wv, lane);
  dma_region(b.unit4, units + 32 * b.B2, 32 * b.B4, wv, lane);
  if (!(b.dbg & 8)) dma_region(b.meta1 + (size_t)tile * b.G * 16, m1s, m1_bytes, wv, lane);
  dma_region(b.meta2 + (size_t)tile * b.S * 16, m2s, m2_bytes, wv, lane);
  if (!(b.dbg & 16)) dma_region(b.otile + (size_t)tile * b.orec_bytes, ots, b.orec_bytes, wv, lane);
  if (!(b.dbg & 4))
    for (int m = 0; m < M; ++m) dma_region(X + (size_t)m * b.K, xs + (size_t)m * rowbytes, 2 * b.K, wv, lane);
  const int nblk = wv < C ? (C - wv + W - 1) / W : 0;  // blocks of this wave
  const int nb0 = nblk < PD ? nblk : PD;               // requested now
  auto block_src = [&](int c) -> const uint4* {
    return c < b.B2 ? b.codes2 + ((size_t)tile * b.B2 + c) * 64 + lane
                    : b.codes4 + ((size_t)tile * b.B4 + (c - b.B2)) * 64 + lane;
  };
#pragma unroll
  for (int r = 0; r < PD; ++r)
    if (r < nb0 && !(b.dbg & 2)) dma16(block_src(wv + r * W), myring + r * 1024);
  wait_vm(nb0);  // the staged operands have landed; the code blocks may still be in flight
  lds_barrier();

  // ---- (2) this wave's blocks, in order
  const unsigned char* xrow0 = xs + (size_t)(i < M ? i : 0) * rowbytes;
  const unsigned char* xrow1 = xs + (size_t)((NT > 1 && i + 16 < M) ? i + 16 : 0) * rowbytes;
  float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  int slot = 0;
  for (int it = 0; it < nblk; ++it) {
    const int c = wv + it * W;
    // Requests of this wave that are younger than block `it` (each freed slot is refilled at
    // once, so PD - 1 blocks follow until the stream runs dry): loads complete in order, hence
    // "at most that many outstanding" means block `it` has landed.
    const int left = nblk - 1 - it;
    if (left >= PD - 1) MPQ_VMCNT(PD - 1); else wait_vm(left);
    uint4 q;
    {
      const uint32_t a =
          (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)(myring + slot * 1024) + lane * 16;
      asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(q) : "v"(a) : "memory");
    }
    if (it + PD < nblk && !(b.dbg & 2)) dma16(block_src(c + PD * W), myring + slot * 1024);
    slot = slot + 1 == PD ? 0 : slot + 1;
    if (b.dbg & 1) { acc0[0] += (float)q.x; continue; }

    const uint2 ue = *(const uint2*)(units + (4 * c + j) * 8);
    const uint32_t m1 = *(const uint16_t*)(m1s + (ue.y & 0xFFFFu) + i * 2);
    const uint32_t m2 = *(const uint32_t*)(m2s + (ue.y >> 16) + i * 4);
    half_t s1 = scale_dequant(m1 & 0xFFu, m2);
    if (ue.x & MPQ_PAD_UNIT) s1 = (half_t)0.0f;
    const half2_t s1p = {s1, s1};
    const half_t zb = bits_to_half((uint16_t)(0x6400u | (m1 >> 8)));  // 1024 + z1
    const uint32_t xo = ue.x & 0x7FFFFFFFu;
    const unsigned char* xb0 = xrow0 + xo;
    const unsigned char* xb1 = xrow1 + xo;
    const uint32_t lo[4] = {q.x, q.y, q.z, q.w};
#define MPQ_MM_STEP(TWO, P)                                                                           \
  {                                                                                                   \
    const uint4 av = decode_step<TWO, P>(lo, hi, s1p, zb, kc);                                        \
    const uint4 bv0 = *(const uint4*)(xb0 + 16 * (P));                                                \
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                    \
                                                  __builtin_bit_cast(half8_t, bv0), acc0, 0, 0, 0);   \
    if (NT > 1) {                                                                                     \
      const uint4 bv1 = *(const uint4*)(xb1 + 16 * (P));                                              \
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                  \
                                                    __builtin_bit_cast(half8_t, bv1), acc1, 0, 0, 0); \
    }                                                                                                 \
  }
    if (c < b.B2) {
      const uint32_t hi[4] = {q.x >> 10, q.y >> 10, q.z >> 10, q.w >> 10};
      MPQ_MM_STEP(true, 0) MPQ_MM_STEP(true, 1) MPQ_MM_STEP(true, 2) MPQ_MM_STEP(true, 3)
      MPQ_MM_STEP(true, 4) MPQ_MM_STEP(true, 5) MPQ_MM_STEP(true, 6) MPQ_MM_STEP(true, 7)
    } else {
      const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
      MPQ_MM_STEP(false, 0) MPQ_MM_STEP(false, 1) MPQ_MM_STEP(false, 2) MPQ_MM_STEP(false, 3)
    }
#undef MPQ_MM_STEP
  }
  // ---- (3) accumulator lane l holds Y[m = l % 16][rows 4*(l/16) .. +3] of this wave's share; the
  //      wave parks it in its own (now idle) ring slots: red[NT][16 m][16 rows]
  float* red = (float*)myring;
  *(float4_t*)(red + i * 16 + 4 * j) = acc0;
  if (NT > 1) *(float4_t*)(red + 256 + i * 16 + 4 * j) = acc1;

  // ---- (4) outliers of row `orow` for batch column om (and om + 16): sum val * X[m][col], all
  //      operands already in LDS (Sec. 4.3, fused: no second kernel, no second trip to memory)
  float oa0 = 0.f, oa1 = 0.f;
  if (b.orec_bytes > 0) {
    const uint32_t* ostart = (const uint32_t*)ots;
    const uint32_t* owords = (const uint32_t*)(ots + MPQ_OTILE_HEAD);
    const int32_t rp0 = (int32_t)ostart[orow], rp1 = (int32_t)ostart[orow + 1];
    const unsigned char* xo0 = xs + (size_t)(om < M ? om : 0) * rowbytes;
    const unsigned char* xo1 = xs + (size_t)((NT > 1 && om + 16 < M) ? om + 16 : 0) * rowbytes;
    auto use = [&](uint32_t word) {
      const uint32_t off = (word & 0xFFFFu) * 2u;
      const float v = (float)bits_to_half((uint16_t)(word >> 16));
      oa0 += v * (float)*(const half_t*)(xo0 + off);
      if (NT > 1) oa1 += v * (float)*(const half_t*)(xo1 + off);
    };
    for (int32_t e = rp0 + oes; e < rp1; e += ostride) use(owords[e]);
    for (int off = Mp; off < 16; off <<= 1) {
      oa0 += __shfl_xor(oa0, off);
      if (NT > 1) oa1 += __shfl_xor(oa1, off);
    }
  }
  __syncthreads();
  {
    const int row = tile * 16 + orow;
    float t0 = oa0, t1 = oa1;
#pragma unroll
    for (int w2 = 0; w2 < W; ++w2) {
      const float* r2 = (const float*)(ring + w2 * (PD * 1024));
      t0 += r2[oq * 16 + orow];
      if (NT > 1) t1 += r2[256 + oq * 16 + orow];
    }
    if (row < b.N) {
      if (oq < M) Y[(size_t)oq * b.N + row] = half_to_bits((half_t)t0);
      if (NT > 1 && oq + 16 < M) Y[(size_t)(oq + 16) * b.N + row] = half_to_bits((half_t)t1);
    }
  }
}

// ------------------------------------------------------------------------------------ dequant
__global__ void __launch_bounds__(256)
mpq_dequant_kernel(const DevBlob b, uint16_t* __restrict__ Wout) {
#pragma clang fp contract(off)
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6, W = blockDim.x >> 6;
  const int i = lane & 15, j = lane >> 4;
  const int C = b.B2 + b.B4;
  const int tile = blockIdx.x;
  const int row = tile * 16 + i;
  const DecodeConsts kc = make_consts();
  for (int c = wv; c < C; c += W) {
    const bool two = c < b.B2;
    const uint4 q = two ? b.codes2[((size_t)tile * b.B2 + c) * 64 + lane]
                        : b.codes4[((size_t)tile * b.B4 + (c - b.B2)) * 64 + lane];
    const uint2 ue = two ? b.unit2[4 * c + j] : b.unit4[4 * (c - b.B2) + j];
    if ((ue.x & MPQ_PAD_UNIT) || row >= b.N) continue;
    const uint32_t m1 = b.meta1[(size_t)tile * b.G * 16 + (ue.y & 0xFFFFu) / 2 + i];
    const uint32_t m2 = b.meta2[(size_t)tile * b.S * 16 + (ue.y >> 16) / 4 + i];
    const half_t s1 = scale_dequant(m1 & 0xFFu, m2);
    const half2_t s1p = {s1, s1};
    const half_t zb = bits_to_half((uint16_t)(0x6400u | (m1 >> 8)));
    uint4* dst = (uint4*)(Wout + (size_t)row * b.K + ue.x / 2);
    const uint32_t lo[4] = {q.x, q.y, q.z, q.w};
    if (two) {
      const uint32_t hi[4] = {q.x >> 10, q.y >> 10, q.z >> 10, q.w >> 10};
      dst[0] = decode_step<true, 0>(lo, hi, s1p, zb, kc);
      dst[1] = decode_step<true, 1>(lo, hi, s1p, zb, kc);
      dst[2] = decode_step<true, 2>(lo, hi, s1p, zb, kc);
      dst[3] = decode_step<true, 3>(lo, hi, s1p, zb, kc);
      dst[4] = decode_step<true, 4>(lo, hi, s1p, zb, kc);
      dst[5] = decode_step<true, 5>(lo, hi, s1p, zb, kc);
      dst[6] = decode_step<true, 6>(lo, hi, s1p, zb, kc);
      dst[7] = decode_step<true, 7>(lo, hi, s1p, zb, kc);
    } else {
      const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
      dst[0] = decode_step<false, 0>(lo, hi, s1p, zb, kc);
      dst[1] = decode_step<false, 1>(lo, hi, s1p, zb, kc);
      dst[2] = decode_step<false, 2>(lo, hi, s1p, zb, kc);
      dst[3] = decode_step<false, 3>(lo, hi, s1p, zb, kc);
    }
  }
}

// W[row][col] = fp16(W[row][col] + val) for every outlier word of the tile (native fp16 add = the
// fp32 add followed by one rounding that the definition states); 16 threads per row.
__global__ void __launch_bounds__(256)
mpq_outlier_add_kernel(const DevBlob b, uint16_t* __restrict__ Wout) {
  const int orow = threadIdx.x >> 4, oq = threadIdx.x & 15;
  const int row = blockIdx.x * 16 + orow;
  if (row >= b.N || b.orec_bytes == 0) return;
  const uint32_t* rec = (const uint32_t*)(b.otile + (size_t)blockIdx.x * b.orec_bytes);
  const uint32_t* words = rec + MPQ_OTILE_HEAD / 4;
  const int32_t rp0 = (int32_t)rec[orow], rp1 = (int32_t)rec[orow + 1];
  for (int32_t e = rp0 + oq; e < rp1; e += 16) {
    const uint32_t word = words[e];
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
  d->unit2 = (const uint2*)(p + h->off_unit2);
  d->unit4 = (const uint2*)(p + h->off_unit4);
  d->codes2 = (const uint4*)(p + h->off_codes2);
  d->codes4 = (const uint4*)(p + h->off_codes4);
  d->meta1 = (const uint16_t*)(p + h->off_meta1);
  d->meta2 = (const uint32_t*)(p + h->off_meta2);
  d->otile = p + h->off_otile;
  d->orec_bytes = h->ocap > 0 ? (int32_t)(MPQ_OTILE_HEAD + 4 * h->ocap) : 0;
  d->N = h->N; d->K = h->K; d->G = h->G; d->S = h->S; d->n2 = h->n2;
  d->U2 = h->U2; d->U4 = h->U4; d->B2 = h->B2; d->B4 = h->B4; d->T = h->T;
  d->nnz = h->nnz;
  d->dbg = 0;
  return MPQ_OK;
}

// Bytes of the `stage` array a batch of M rows needs (unit tables, the tile's meta words, activations).
size_t stage_bytes(const MpqHeader& h, int M) {
  const size_t orec = h.ocap > 0 ? MPQ_OTILE_HEAD + 4 * h.ocap : 0;
  return 32ull * (h.B2 + h.B4) + 32ull * h.G + 64ull * h.S + orec + (size_t)M * (2ull * h.K + 16);
}

int g_ring_depth = 0;  // 0 = automatic
int g_dbg = 0;

template <int NT, int PD, int STB>
mpq_status launch_mm(const MpqHeader& h, const DevBlob& d, const uint16_t* X, uint16_t* Y, int M, hipStream_t s) {
  DevBlob dd = d;
  dd.dbg = g_dbg;
  hipLaunchKernelGGL((mpq_mm_kernel<NT, PD, STB>), dim3(h.T), dim3(256), 0, s, dd, X, Y, M);
  return hipGetLastError() == hipSuccess ? MPQ_OK : MPQ_ERR_HIP;
}

// Static LDS size classes of the product kernel (bytes of `stage`); the ring depth per class
// keeps several workgroups resident per compute unit (160 KiB of LDS).
template <int NT>
mpq_status mm_chunk(const MpqHeader& h, const DevBlob& d, const uint16_t* X, uint16_t* Y, int M, hipStream_t s) {
  const size_t need = stage_bytes(h, M);
  const int pd = g_ring_depth;
  if (need <= 13312) {
    if (pd == 2) return launch_mm<NT, 2, 13312>(h, d, X, Y, M, s);
    if (pd == 4) return launch_mm<NT, 4, 13312>(h, d, X, Y, M, s);
    if (pd == 5) return launch_mm<NT, 5, 13312>(h, d, X, Y, M, s);
    return launch_mm<NT, 3, 13312>(h, d, X, Y, M, s);
  }
  if (need <= 24 * 1024) return launch_mm<NT, 4, 24 * 1024>(h, d, X, Y, M, s);
  if (need <= 40 * 1024) return launch_mm<NT, 4, 40 * 1024>(h, d, X, Y, M, s);
  if (need <= 80 * 1024) return launch_mm<NT, 4, 80 * 1024>(h, d, X, Y, M, s);
  if (need <= 144 * 1024) return launch_mm<NT, 3, 144 * 1024>(h, d, X, Y, M, s);
  return MPQ_ERR_UNSUPPORTED;
}

mpq_status mm_all(const MpqHeader& h, const DevBlob& d, const uint16_t* X, uint16_t* Y, int M, hipStream_t s) {
  constexpr size_t kStageMax = 144 * 1024;
  if (stage_bytes(h, 1) > kStageMax) return MPQ_ERR_UNSUPPORTED;
  int Mc = M;  // largest batch chunk whose activations fit LDS together with the tables
  while (Mc > 1 && stage_bytes(h, Mc) > kStageMax) --Mc;
  if (Mc > 16 && Mc < M) Mc = 16;
  for (int m0 = 0; m0 < M; m0 += Mc) {
    const int mc = M - m0 < Mc ? M - m0 : Mc;
    const uint16_t* Xc = X + (size_t)m0 * h.K;
    uint16_t* Yc = Y + (size_t)m0 * h.N;
    mpq_status st = mc > 16 ? mm_chunk<2>(h, d, Xc, Yc, mc, s) : mm_chunk<1>(h, d, Xc, Yc, mc, s);
    if (st != MPQ_OK) return st;
  }
  return MPQ_OK;
}

}  // namespace

extern "C" {

// Tuning hook for sweeps; not part of the supported interface and not thread safe.
// key 0: ring depth (code blocks in flight per wave) for the smallest LDS class, 0 = automatic.
void mpq_debug_set(int key, int value) {
  if (key == 0) g_ring_depth = value;
  if (key == 1) g_dbg = value;
}

mpq_status mpq_gemm(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev, uint16_t* Y_dev,
                    int32_t M, void* stream) {
  if (!X_dev || !Y_dev) return MPQ_ERR_NULL;
  if (M < 1 || M > MPQ_MAX_M) return MPQ_ERR_SHAPE;
  MpqHeader h;
  DevBlob d;
  mpq_status st = make_dev(hdr_host, blob_dev, &h, &d);
  if (st != MPQ_OK) return st;
  if ((((uintptr_t)X_dev | (uintptr_t)Y_dev) & 15u) != 0) return MPQ_ERR_ALIGN;
  return mm_all(h, d, X_dev, Y_dev, M, (hipStream_t)stream);
}

mpq_status mpq_gemv(const void* hdr_host, const void* blob_dev, const uint16_t* x_dev, uint16_t* y_dev,
                    void* stream) {
  return mpq_gemm(hdr_host, blob_dev, x_dev, y_dev, 1, stream);
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
  hipLaunchKernelGGL(mpq_dequant_kernel, dim3(h.T), dim3(256), 0, s, d, W_out_dev);
  if (hipGetLastError() != hipSuccess) return MPQ_ERR_HIP;
  if (add_outliers && h.nnz > 0) {
    hipLaunchKernelGGL(mpq_outlier_add_kernel, dim3(h.T), dim3(256), 0, s, d, W_out_dev);
    if (hipGetLastError() != hipSuccess) return MPQ_ERR_HIP;
  }
  return MPQ_OK;
}

}  // extern "C"
