// mpq_kernels.hip - gfx950 kernels and device entry points of the mixed-precision weight library.
//
// Kernels (all read the packed blob described in mpq_format.h):
//   mpq_gemv_kernel      Algorithm 1 (GEMV with asynchronous dequantization) re-designed for CDNA4,
//                        with the outlier product of Sec. 4.3 fused in as a per-row correction.
//   mpq_mm_kernel        the same product for a batch of 2..32 activation rows that fit the LDS.
//   mpq_mms_kernel       the same for batches that do not: one K-range of the activations resident
//                        per workgroup, partial sums added up by mpq_mms_finish_kernel.
//   mpq_dequant_kernel, mpq_dequant_lines_kernel   eq. 5 applied twice (scale, then weight), written out as row-major fp16.
//   mpq_outlier_add_kernel  adds the CSR values to a dequantized matrix (dense + sparse, Sec. 2.3).
//
// Mapping shared by the kernels.  A wavefront load of 1 KiB is one block: lane = j*16 + i holds the
// 16-byte unit j (of 4) of row i (of a 16-row tile).  The blocks of a tile, first the 2-bit stream,
// then the 4-bit stream, go round-robin to the waves that work on the tile.  A lane therefore
// always decodes codes of ONE row and ONE first-order group, so the group's scale and zero point
// are per-lane scalars.
//
// Per-weight arithmetic (bit-exact to the definition in mpq.h):
//   a mask isolates two codes (low / high half-word of a dword); OR-ing 0x6400 into each half
//   makes the fp16 numbers 1024 + c*2^o; one packed fma (x 2^-o, - (1024*2^-o + z1)) gives the
//   exact integers c - z1; one packed fp16 multiply by s1 is the rounding the definition asks
//   for.  The product kernel hands the resulting pairs to the matrix core.
#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdint.h>
#include <string.h>


#include "../../include/mpq.h"
#include "mpq_format.h"

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// Phase stamps of the timeline build (-DMPQ_TIMELINE, a second library next to the product): wall-clock
// reads (s_memrealtime, 100 MHz) at the phase boundaries of the batch-1 kernels.  The first and the last
// wave of every workgroup write theirs to a buffer of 2 x 16 words per workgroup that the measuring
// program hands over with mpq_timeline_buffer.  The product build compiles all of it away.
#ifdef MPQ_TIMELINE
__device__ unsigned long long* mpq_timeline_buf;
#define MPQ_TL_DECL unsigned long long tl_[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#define MPQ_STAMP(k) tl_[k] = __builtin_amdgcn_s_memrealtime();
#define MPQ_TL_NOTE(k, v) tl_[k] = (unsigned long long)(v);
#define MPQ_TL_FLUSH(WG, WAVE, LASTWAVE, LANE)                                                          \
  if (mpq_timeline_buf && (LANE) == 0 && ((WAVE) == 0 || (WAVE) == (LASTWAVE))) {                      \
    unsigned long long* o_ = mpq_timeline_buf + ((size_t)(WG) * 2 + ((WAVE) == 0 ? 0 : 1)) * 16;        \
    _Pragma("unroll") for (int q_ = 0; q_ < 16; ++q_) o_[q_] = tl_[q_];                                 \
  }
#else
#define MPQ_TL_DECL
#define MPQ_STAMP(k)
#define MPQ_TL_NOTE(k, v)
#define MPQ_TL_FLUSH(WG, WAVE, LASTWAVE, LANE)
#endif

struct DevBlob {
  const unsigned char* tiles;  // first tile record
  const unsigned char* units;  // unit table (2-bit units, then 4-bit units), 8 bytes per unit
  uint32_t tile_stride;        // bytes between tile records
  uint32_t side_bytes;         // meta1 | meta2 | outlier record at the head of a tile record
  uint32_t codes_off;          // offset of the code blocks inside a tile record
  uint32_t off_m2, off_ot;     // offsets of meta2 and of the outlier record inside the side part
  uint32_t m2_shift;           // lane part of a meta2 address = 4 * (row >> m2_shift)
  uint32_t off_m1b, off_s2, off_z2;  // aligned metadata (Sec. 3.3): bytes of the 4-bit groups, second-order scales, zeros
  uint32_t pad_entry;                // bits 16-31 of the table word of a padding piece (the zero second-order entry)
  uint32_t off_oidx, ocap;           // outlier block index inside a tile record (0 = none); words per outlier record
  int32_t N, K, G, S, B2, C, T;
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
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "do not wait").  Larger n wait for vmcnt(15),
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
    case 9: MPQ_VMCNT(9); break;
    case 10: MPQ_VMCNT(10); break;
    case 11: MPQ_VMCNT(11); break;
    case 12: MPQ_VMCNT(12); break;
    case 13: MPQ_VMCNT(13); break;
    case 14: MPQ_VMCNT(14); break;
    default: MPQ_VMCNT(15); break;
  }
}

// The same for 0 <= n <= MAXN known at compile time to be small: two compares instead of the switch.
template <int MAXN>
__device__ __forceinline__ void wait_vm_upto(int n) {
  if (MAXN <= 2) {
    if (n >= 2) MPQ_VMCNT(2);
    else if (n == 1) MPQ_VMCNT(1);
    else MPQ_VMCNT(0);
  } else {
    wait_vm(n);
  }
}

// The product kernel issues its global loads with inline asm and waits for them with explicit
// s_waitcnt vmcnt(n): the compiler's own wait insertion cannot count requests issued in loops and
// would otherwise wait for ALL outstanding loads (vmcnt(0)) whenever LDS written by a direct load
// is read, which serialises the whole pipeline.  Values loaded this way must not be used before
// the matching wait_vm().

// 16 bytes per lane straight from global memory into LDS (no register staging): lane l reads
// gbase + voff(l) and writes LDS byte lds + 16*l.  gbase and lds are wave-uniform and live in
// scalar registers, so the address arithmetic of the caller stays on the scalar unit.
__device__ __forceinline__ void dma16(const unsigned char* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(gbase)
               : "memory");
}

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)p;
}

// Copies `bytes` (a multiple of 16) from gbase to LDS byte address lds; the NW waves of the
// workgroup take 1 KiB pieces in turn.  lane16 = 16 * lane.
template <uint32_t NW>
__device__ __forceinline__ void dma_linear(const unsigned char* gbase, uint32_t lds, uint32_t bytes, uint32_t wv,
                                           uint32_t lane16) {
  // one form for whole and partial pieces: the lanes beyond the end are masked off (fewer instructions than a
  // branch between the two, and these run in the prologue of every wave)
  for (uint32_t off = wv * 1024u; off < bytes; off += NW * 1024u)
    if (off + lane16 < bytes) dma16(gbase + off, lane16, lds + off);
}

// Second-order dequantization of a first-order scale: fp16((fp32(s_int) - fp32(z2)) * fp32(s2)).
// (Algorithm 1, second-order dequantization step; eq. 5 form.)
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

// The same where the second-order zero is stored as an integer 0..15 (aligned metadata, Sec. 3.3 "Zero Padding"):
// s_int and z2 are small integers, so fp32(s_int) - fp32(z2) is the integer difference converted once.
__device__ __forceinline__ half_t scale_dequant_int_zero(uint32_t s_int, uint32_t z2, uint32_t s2_bits) {
#pragma clang fp contract(off)
  const float t = (float)((int32_t)s_int - (int32_t)z2);
  float u = t * (float)bits_to_half((uint16_t)s2_bits);
  asm volatile("" : "+v"(u));  // two roundings, as in scale_dequant
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
  uint32_t mask2[4], mask4[2], sc2[4], sc4[2];
  uint32_t magic;
};

__device__ __forceinline__ DecodeConsts make_consts() {
  DecodeConsts k;
  // 2-bit fields sit at bit offsets 1, 3, 5, 7 of a half-word (mpq_format.h)
  k.mask2[0] = sgpr_const(0x00060006u); k.mask2[1] = sgpr_const(0x00180018u);
  k.mask2[2] = sgpr_const(0x00600060u); k.mask2[3] = sgpr_const(0x01800180u);
  k.mask4[0] = sgpr_const(0x000F000Fu); k.mask4[1] = sgpr_const(0x00F000F0u);
  k.sc2[0] = sgpr_const(0x38003800u);  // 1/2
  k.sc2[1] = sgpr_const(0x30003000u);  // 1/8
  k.sc2[2] = sgpr_const(0x28002800u);  // 1/32
  k.sc2[3] = sgpr_const(0x20002000u);  // 1/128
  k.sc4[0] = sgpr_const(0x3C003C00u);  // 1
  k.sc4[1] = sgpr_const(0x2C002C00u);  // 1/16
  asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(k.magic));  // fp16 1024.0 in both halves
  return k;
}

__device__ __forceinline__ uint32_t rotr8(uint32_t v) { return __builtin_amdgcn_alignbit(v, v, 8); }

// First-order dequantization (eq. 5) of step P of a unit: the four dwords give the four fp16 pairs
// of columns 8P .. 8P+7.  TWO_BIT selects 2-bit (P = 0..7) or 4-bit (P = 0..3) fields.
// zb = fp16(1024 + z1); lo = the unit's dwords, hi = the same rotated right by 8 (2-bit) or shifted
// right by 8 (4-bit), so that every field sits in mantissa bits of its half-word: a 2-bit field of
// step P is at bit offset (P < 4 ? 1 : 3) + 4 (P % 2) of lo (P % 4 < 2) or hi; a 4-bit field at
// offset 4 (P % 2) of lo (P < 2) or hi.
template <bool TWO_BIT, int P>
__device__ __forceinline__ uint4 decode_step(const uint32_t (&lo)[4], const uint32_t (&hi)[4], const half2_t s1p,
                                             const half_t zb, const DecodeConsts& kc) {
#pragma clang fp contract(off)
  constexpr int pp = TWO_BIT ? (P < 4 ? 0 : 1) + 2 * (P & 1) : (P & 1);
  constexpr bool shifted = TWO_BIT ? ((P & 3) >= 2) : (P >= 2);
  // 1024 - 1024 * f with f = 2^-offset of the field: off - zb = -(1024 * f + z1), exact, below 2048
  constexpr float off = TWO_BIT ? (pp == 0 ? 512.f : pp == 1 ? 896.f : pp == 2 ? 992.f : 1016.f)
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

// Scale, zero point and activation offset of the NP pieces of a unit (one piece per first-order
// group that the unit touches; one piece for g1 >= 64).  ue points at the unit's table entries.
// The same from unit table entries that were fetched earlier.
template <int NP>
__device__ __forceinline__ void finish_pieces(const uint2 (&ent)[NP], const unsigned char* m1i, const unsigned char* m2i,
                                              half2_t (&s1p)[NP], half_t (&zb)[NP], uint32_t (&xoff)[NP]) {
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const uint2 e = ent[q];
    const uint32_t m1 = *(const uint16_t*)(m1i + (e.y & 0xFFFFu));
    const uint32_t m2 = *(const uint32_t*)(m2i + (e.y >> 16));
    const half_t s1 = scale_dequant(m1 & 0xFFu, m2);  // exactly 0 for a padding piece (zero meta entries)
    s1p[q] = half2_t{s1, s1};
    zb[q] = bits_to_half((uint16_t)(0x6400u | (m1 >> 8)));  // 1024 + z1
    xoff[q] = e.x;
  }
}

// The same for the aligned metadata of Sec. 3.3 ("Memory Alignment"): a 2-bit piece finds its 2-bit zero
// point and its 4- or 3-bit scale in the 16-bit word that three consecutive 2-bit groups of the row share
// (zero points at bits 0-5, scales at bits 6, 10, 13), a 4-bit piece both in one byte; the second-order zero
// is an integer in a byte next to the fp16 second-order scale.  `side` = the tile's side part, row = 0..15.
template <int NP, bool FOUR>
__device__ __forceinline__ void pieces_aligned(const uint2 (&ent)[NP], const unsigned char* side, const DevBlob& b,
                                               const uint32_t row, half2_t (&s1p)[NP], half_t (&zb)[NP], uint32_t (&xoff)[NP]) {
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const uint2 e = ent[q];
    uint32_t s_int, z1;
    if (FOUR) {
      const uint32_t w = *(const uint8_t*)(side + b.off_m1b + (e.y & 0xFFFFu) + row);
      s_int = w & 15u;
      z1 = w >> 4;
    } else {
      const uint32_t pos = e.y & 3u;
      const uint32_t w = *(const uint16_t*)(side + (e.y & 0xFFFCu) + 2u * row);
      z1 = (w >> (2u * pos)) & 3u;
      s_int = pos == 0 ? (w >> 6) & 15u : (w >> (pos == 1 ? 10u : 13u)) & 7u;
    }
    const uint32_t idx = (e.y >> 16) + (row >> b.m2_shift);
    const uint32_t s2 = *(const uint16_t*)(side + b.off_s2 + 2u * idx);
    const uint32_t z2 = *(const uint8_t*)(side + b.off_z2 + idx);  // 0..15
    const half_t s1 = scale_dequant_int_zero(s_int, z2, s2);       // exactly 0 for a padding piece
    s1p[q] = half2_t{s1, s1};
    zb[q] = bits_to_half((uint16_t)(0x6400u | z1));  // 1024 + z1
    xoff[q] = e.x;
  }
}

template <int NP>
__device__ __forceinline__ void load_pieces(const unsigned char* ue, const unsigned char* m1i, const unsigned char* m2i,
                                            half2_t (&s1p)[NP], half_t (&zb)[NP], uint32_t (&xoff)[NP]) {
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const uint2 e = *(const uint2*)(ue + 8 * q);
    const uint32_t m1 = *(const uint16_t*)(m1i + (e.y & 0xFFFFu));
    const uint32_t m2 = *(const uint32_t*)(m2i + (e.y >> 16));
    const half_t s1 = scale_dequant(m1 & 0xFFu, m2);  // exactly 0 for a padding piece (zero meta entries)
    s1p[q] = half2_t{s1, s1};
    zb[q] = bits_to_half((uint16_t)(0x6400u | (m1 >> 8)));  // 1024 + z1
    xoff[q] = e.x;
  }
}

// ------------------------------------------------------------------------------------ product
//
// Y[m][n] = sum_k X[m][k] W[n][k] + outliers, 2 <= M <= 16*NT.  Persistent workgroups of WV
// waves: workgroup g handles the 16-row tiles g, g + grid, g + 2*grid, ...
//
// Data movement (the "asynchronous dequantization" of Sec. 5 on this hardware).  Every global
// load of the kernel is a direct global->LDS load (global_load_lds_dwordx4, no registers):
//   - once per workgroup: the activations (one LDS row per batch row) and the unit tables;
//   - once per tile, one tile ahead: the tile's side record (scale words + outlier record) into one
//     of two buffers;
//   - continuously: the code blocks.  Each wave owns PD ring slots of 1 KiB and walks its own
//     sequence of blocks (its share of tile g, then of tile g + grid, ...).  A consumed slot is
//     refilled at once with the next block of the sequence, across tile boundaries, so PD blocks per
//     wave are in flight from the first instruction to the last.
// Loads complete in order, so "block is there" is s_waitcnt vmcnt(number of younger requests of this
// wave): PD - 1 in steady state.  The second-order scale of a block is reconstructed while the
// later blocks are on their way.  The waits are written by hand (inline asm loads are invisible to
// the compiler's own wait insertion, which cannot count requests issued in loops and would wait
// for ALL outstanding loads before every LDS read).
//
// Compute: the decoded fp16 weights of a block are exactly the A operand of
// v_mfma_f32_16x16x32_f16 (lane j*16+i holds 8 consecutive columns of row i), the activations of
// the same columns are the B operand (lane j*16+m holds X[m][same 8 columns]), and the 16x16 fp32
// accumulator holds Y[m][row] for the whole tile.  The matrix core does the multiply-accumulate
// and the reduction over the four unit columns, so the vector ALU only decodes.  Batch columns
// beyond M compute garbage that is never stored.
//
// Two barriers per tile: one before a tile's side record is read (every wave has waited for its
// own share of that record), one before the waves' accumulators are summed.
//
// WV = waves per workgroup (4, 8 or 16), all working on the same tile.  More waves per tile fill
// the 32 wave slots of a compute unit with fewer workgroups (less LDS for staged operands per
// wave) and keep every SIMD busy when the matrix has few row tiles (4096 rows = 256 tiles = one
// tile per compute unit).
template <int NT, int PD, int LDSB, int WV = 4, int PU = 1, bool AL = false>
__global__ void __launch_bounds__(WV * 64)
mpq_mm_kernel(const DevBlob b, const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, const int M) {
#pragma clang fp contract(off)
  static_assert(PD >= 1 && PD <= 8, "ring depth");
  __shared__ __align__(16) unsigned char lds[LDSB];
  constexpr uint32_t W = WV;
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t i = lane & 15u, j = lane >> 4, lane16 = lane * 16u;
  const uint32_t C = b.C, T = b.T, grid = gridDim.x;
  // LDS layout: ring | reduction slots | side record x 2 | unit table | activation rows
  constexpr int PU4 = PU > 1 ? PU / 2 : 1;   // pieces per 2-bit unit (PU) and per 4-bit unit
  const uint32_t units_bytes = 32u * PU * C;
  const uint32_t rowbytes = 2u * b.K + 16u;  // + 16: rows of a batch start in different LDS banks
  unsigned char* const ring = lds;
  unsigned char* const side0 = lds + W * PD * 1024 + W * NT * 1024;
  unsigned char* const units = side0 + 2 * b.side_bytes;
  unsigned char* const xs = units + units_bytes;
  const DecodeConsts kc = make_consts();

  // ---- (1) requests of the first tile, oldest first: staged operands, then this wave's code blocks
  const uint32_t tile0 = blockIdx.x;
  const unsigned char* tileptr = b.tiles + (size_t)tile0 * b.tile_stride;
  const size_t tilestep = (size_t)grid * b.tile_stride;
  dma_linear<W>(tileptr, lds_addr(side0), b.side_bytes, wv, lane16);
  dma_linear<W>(b.units, lds_addr(units), units_bytes, wv, lane16);
  for (int m = 0; m < M; ++m)
    dma_linear<W>((const unsigned char*)(X + (size_t)m * b.K), lds_addr(xs) + m * rowbytes, 2u * b.K, wv, lane16);
  // this wave's sequence of blocks: (tile0, wv), (tile0, wv + 4), ..., (tile0 + grid, wv), ...
  const uint32_t ring0 = lds_addr(ring) + wv * (PD * 1024);
  const unsigned char* rbase = tileptr + b.codes_off;  // code blocks of the tile being requested
  uint32_t rtile = wv < C ? tile0 : T;                 // T = nothing left to request
  uint32_t rc = wv;
  uint32_t inflight = 0;
#pragma unroll
  for (uint32_t r = 0; r < PD; ++r) {
    if (rtile < T) {
      dma16(rbase + rc * 1024u, lane16, ring0 + r * 1024u);
      ++inflight;
      rc += W;
      if (rc >= C) { rc = wv; rtile += grid; rbase += tilestep; }
    }
  }
  wait_vm_upto<PD>((int)inflight);  // the staged operands have landed; the code blocks may still be in flight
  lds_barrier();

  const unsigned char* xrow0 = xs + (i < (uint32_t)M ? i : 0u) * rowbytes;
  const unsigned char* xrow1 = xs + ((NT > 1 && i + 16 < (uint32_t)M) ? i + 16 : 0u) * rowbytes;
  const unsigned char* unitj = units + j * (8 * PU);
  const uint32_t ringl = ring0 + lane16;
  // outlier / output mapping: 16 consecutive lanes share row `orow`; lane q takes batch column
  // q % Mp (and + 16) and every (16/Mp)-th word of the row
  const uint32_t orow = tid >> 4, oq = tid & 15u;
  uint32_t Mp = 1;
  while (Mp < (uint32_t)M && Mp < 16) Mp <<= 1;
  const uint32_t om = oq & (Mp - 1), oes = oq / Mp, ostride = 16 / Mp;
  const unsigned char* xo0 = xs + (om < (uint32_t)M ? om : 0u) * rowbytes;
  const unsigned char* xo1 = xs + ((NT > 1 && om + 16 < (uint32_t)M) ? om + 16 : 0u) * rowbytes;

  uint32_t slot = 0;        // ring slot of the next block to consume
  uint32_t since_side = 0;  // requests of this wave issued after its share of the next side record
  uint32_t par = 0;
  for (uint32_t tile = tile0; tile < T; tile += grid, par ^= 1u) {
    const unsigned char* side = side0 + par * b.side_bytes;
    if (tile != tile0) {
      wait_vm((int)since_side);  // this wave's share of the side record has landed
      lds_barrier();             // ... and everybody else's; everybody is done with the previous tile
    }
    tileptr += tilestep;
    if (tile + grid < T) dma_linear<W>(tileptr, lds_addr(side0 + (par ^ 1u) * b.side_bytes), b.side_bytes, wv, lane16);
    since_side = 0;
    const unsigned char* m1i = side + i * 2;
    const unsigned char* m2i = side + b.off_m2 + (i >> b.m2_shift) * 4;

    // ---- (2) this wave's blocks of the tile, in order
    float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#define MPQ_MM_STEP(TWO, P)                                                                           \
  {                                                                                                   \
    constexpr int SPP = ((TWO) ? 8 : 4) / ((TWO) ? PU : PU4), Q = (P) / SPP, PO = (P) % SPP;          \
    const uint4 av = decode_step<TWO, P>(lo, hi, s1p[Q], zb[Q], kc);                                  \
    const uint4 bv0 = *(const uint4*)(xrow0 + xoff[Q] + 16 * PO);                                     \
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                    \
                                                  __builtin_bit_cast(half8_t, bv0), acc0, 0, 0, 0);   \
    if (NT > 1) {                                                                                     \
      const uint4 bv1 = *(const uint4*)(xrow1 + xoff[Q] + 16 * PO);                                   \
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                  \
                                                    __builtin_bit_cast(half8_t, bv1), acc1, 0, 0, 0); \
    }                                                                                                 \
  }
// Fetch of the next block of this wave (wait, read its ring slot, refill the slot) and the
// per-piece set-up; the 2-bit blocks of a tile come first in the wave's sequence, then the 4-bit ones.
#define MPQ_MM_BLOCK_HEAD(NP, FOUR)                                                                    \
  /* Requests younger than the block needed now: the other blocks in flight (stricter than            \
     necessary when a side-record request sits between them, never laxer). */                         \
  if (inflight == PD) MPQ_VMCNT(PD - 1); else if (PD == 2) MPQ_VMCNT(0); else wait_vm((int)inflight - 1); \
  uint4 q;                                                                                            \
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(q) : "v"(ringl + slot * 1024u) : "memory"); \
  --inflight;                                                                                         \
  if (rtile < T) { /* refill the freed slot with the next block of this wave's sequence */            \
    dma16(rbase + rc * 1024u, lane16, ring0 + slot * 1024u);                                          \
    ++inflight;                                                                                       \
    ++since_side;                                                                                     \
    rc += W;                                                                                          \
    if (rc >= C) { rc = wv; rtile += grid; rbase += tilestep; }                                       \
  }                                                                                                   \
  slot = slot + 1 == PD ? 0 : slot + 1;                                                               \
  half2_t s1p[NP];                                                                                    \
  half_t zb[NP];                                                                                      \
  uint32_t xoff[NP];                                                                                  \
  if constexpr (AL) {                                                                                 \
    uint2 ent[NP];                                                                                    \
    _Pragma("unroll") for (int qq = 0; qq < NP; ++qq) ent[qq] = *(const uint2*)(unitj + c * (32u * PU) + 8 * qq); \
    pieces_aligned<NP, FOUR>(ent, side, b, i, s1p, zb, xoff);                                         \
  } else {                                                                                            \
    load_pieces<NP>(unitj + c * (32u * PU), m1i, m2i, s1p, zb, xoff);                                 \
  }                                                                                                   \
  const uint32_t lo[4] = {q.x, q.y, q.z, q.w};
    uint32_t c = wv;
    for (; c < (uint32_t)b.B2; c += W) {
      MPQ_MM_BLOCK_HEAD(PU, false)
      const uint32_t hi[4] = {rotr8(q.x), rotr8(q.y), rotr8(q.z), rotr8(q.w)};
      MPQ_MM_STEP(true, 0) MPQ_MM_STEP(true, 1) MPQ_MM_STEP(true, 2) MPQ_MM_STEP(true, 3)
      MPQ_MM_STEP(true, 4) MPQ_MM_STEP(true, 5) MPQ_MM_STEP(true, 6) MPQ_MM_STEP(true, 7)
    }
    for (; c < C; c += W) {
      MPQ_MM_BLOCK_HEAD(PU4, true)
      const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
      MPQ_MM_STEP(false, 0) MPQ_MM_STEP(false, 1) MPQ_MM_STEP(false, 2) MPQ_MM_STEP(false, 3)
    }
#undef MPQ_MM_BLOCK_HEAD
#undef MPQ_MM_STEP
    // ---- (3) accumulator lane l holds Y[m = l % 16][rows 4*(l/16) .. +3] of this wave's share:
    //      red[wave][NT][16 m][16 rows]
    constexpr uint32_t red_stride = NT * 1024;  // bytes between waves
    unsigned char* const red = lds + W * PD * 1024;
    float* myred = (float*)(red + wv * red_stride);
    *(float4_t*)(myred + i * 16 + 4 * j) = acc0;
    if (NT > 1) *(float4_t*)(myred + 256 + i * 16 + 4 * j) = acc1;

    // ---- (4) outliers (Sec. 4.3, fused: no second kernel, no second trip to memory); all operands
    //      are already in LDS
    float oa0 = 0.f, oa1 = 0.f;
    if (WV == 4 || wv < 4) {  // the first 256 threads cover the 16 rows
      const uint32_t* ostart = (const uint32_t*)(side + b.off_ot);
      const uint32_t* owords = ostart + MPQ_OTILE_HEAD / 4;
      const uint32_t rp0 = ostart[orow], rp1 = ostart[orow + 1];
      // four words per lane in flight: the chain word -> activation is two LDS round trips, and the other
      // waves of the workgroup wait at the barrier below meanwhile (a word beyond the row's end counts as
      // value 0 at column 0).  Sharing the words between all waves of the workgroup was measured too:
      // 3 us per Llama2-7B layer faster at 1.5 % outliers and M = 4, 1 us slower at 0 and 0.5 %.
      for (uint32_t e = rp0 + oes; e < rp1; e += 4u * ostride) {
        uint32_t word[4];
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) word[u] = e + u * ostride < rp1 ? owords[e + u * ostride] : 0u;
        half_t x0[4], x1[4];
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
          x0[u] = *(const half_t*)(xo0 + (word[u] & 0xFFFFu) * 2u);
          if (NT > 1) x1[u] = *(const half_t*)(xo1 + (word[u] & 0xFFFFu) * 2u);
        }
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
          const float v = (float)bits_to_half((uint16_t)(word[u] >> 16));
          oa0 += v * (float)x0[u];
          if (NT > 1) oa1 += v * (float)x1[u];
        }
      }
      for (uint32_t off = Mp; off < 16; off <<= 1) {
        oa0 += __shfl_xor(oa0, off);
        if (NT > 1) oa1 += __shfl_xor(oa1, off);
      }
    }
    lds_barrier();
    if (WV == 4 || wv < 4) {
      const uint32_t row = tile * 16 + orow;
      float t0 = oa0, t1 = oa1;
#pragma unroll
      for (uint32_t w2 = 0; w2 < W; ++w2) {
        const float* r2 = (const float*)(red + w2 * red_stride);
        t0 += r2[oq * 16 + orow];
        if (NT > 1) t1 += r2[256 + oq * 16 + orow];
      }
      if (row < (uint32_t)b.N) {
        if (oq < (uint32_t)M) Y[(size_t)oq * b.N + row] = half_to_bits((half_t)t0);
        if (NT > 1 && oq + 16 < (uint32_t)M) Y[(size_t)(oq + 16) * b.N + row] = half_to_bits((half_t)t1);
      }
    }
  }
}

// ------------------------------------------------------------------------------------ product, large batches
//
// Y = X W^T for batches whose activations do not fit the LDS next to everything else (M * K * 2
// bytes above roughly 100 KiB), with the weights read and decoded once whatever M is:
//
//   The code blocks of a tile are cut into H ranges in stream order (range h = an H-th of the 2-bit
//   blocks and an H-th of the 4-bit blocks, sizes differing by at most one) and the tiles into NB
//   bands.  Workgroup (h, band) gathers the activations of range h into LDS ONCE, in the order the
//   blocks use them: slot ((unit*8 + step) * XR + m) holds the 8 fp16 values
//   X[m][k0(unit) + 8*step ..], XR = 8, 16 or 32 staged batch rows, so the B operand of a step is
//   linear in (block, unit, step).  It then walks the band's tiles in groups of up to R = 8,
//   decoding only the blocks of its range.  The blocks of a group, in the order (position in the
//   range, tile), are split between the waves in contiguous pieces, so that a wave reads the B
//   operands of a position from LDS once for all tiles of the group; it keeps one accumulator per
//   tile in registers.  The ring of code blocks stays full from the first tile of the band to the
//   last.
//
//   The first-order (s_int, z1) and second-order (s2, z2) words of a block travel with it: after
//   the 1 KiB of codes, one dword per lane and piece that holds the lane's meta1 entry and one that
//   holds its meta2 entry, gathered through the unit table, land in the same ring slot (1.5 KiB
//   and three direct loads per block for g1 >= 64; 1 KiB + 512 B and 1 + 2 loads per piece of a
//   unit for shorter groups), so no per-tile side record is staged and no barrier separates tiles.
//
//   After a group of tiles the waves park their accumulators, meet, and every (row, batch column)
//   is summed over the waves in a fixed order and written as fp32 to P[h][tile][column][row].  A
//   second kernel adds the H partial sums in order, adds the outlier product of the row (Sec. 4.3)
//   and rounds to fp16: results are bit-identical from run to run.
struct SlicePlan {
  int32_t H, NB, R;
  uint32_t older16;  // sixteenths of a SIMD's blocks that go to the older of its two waves
  uint32_t off_units, off_park, off_xbuf;  // LDS byte offsets (ring at 0)
};

__device__ __forceinline__ void dma4(const unsigned char* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds), "v"(voff), "s"(gbase)
               : "memory");
}

// Reads a ring slot of the large-batch kernel: the 16 bytes of codes of the lane and the first NP of
// its PUV (meta1, meta2) dword pairs, which sit at byte 1024 + 256 q and 1024 + 256 (PUV + q) of the
// slot.  Reads and wait are ONE asm statement: anything the compiler places between a read and the
// wait (a register copy, say) would see the register before the data has arrived.
template <int NP, int PUV>
__device__ __forceinline__ void ring_read(uint32_t code_addr, uint32_t meta_addr, uint4& q, uint32_t (&w1)[NP],
                                          uint32_t (&w2)[NP]) {
  static_assert(NP == 1 || NP == 2 || NP == 4, "pieces per unit");
  constexpr int O2 = 256 * PUV;  // meta2 words follow the PUV meta1 words
  if constexpr (NP == 1) {
    asm volatile("ds_read_b128 %0, %3\n\tds_read_b32 %1, %4\n\tds_read_b32 %2, %4 offset:%5\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(q), "=&v"(w1[0]), "=&v"(w2[0])
                 : "v"(code_addr), "v"(meta_addr), "i"(O2)
                 : "memory");
  } else if constexpr (NP == 2) {
    asm volatile("ds_read_b128 %0, %5\n\tds_read_b32 %1, %6\n\tds_read_b32 %2, %6 offset:256\n\t"
                 "ds_read_b32 %3, %6 offset:%7\n\tds_read_b32 %4, %6 offset:%8\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(q), "=&v"(w1[0]), "=&v"(w1[1]), "=&v"(w2[0]), "=&v"(w2[1])
                 : "v"(code_addr), "v"(meta_addr), "i"(O2), "i"(O2 + 256)
                 : "memory");
  } else {
    asm volatile("ds_read_b128 %0, %9\n\tds_read_b32 %1, %10\n\tds_read_b32 %2, %10 offset:256\n\t"
                 "ds_read_b32 %3, %10 offset:512\n\tds_read_b32 %4, %10 offset:768\n\t"
                 "ds_read_b32 %5, %10 offset:%11\n\tds_read_b32 %6, %10 offset:%12\n\t"
                 "ds_read_b32 %7, %10 offset:%13\n\tds_read_b32 %8, %10 offset:%14\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(q), "=&v"(w1[0]), "=&v"(w1[1]), "=&v"(w1[2]), "=&v"(w1[3]), "=&v"(w2[0]), "=&v"(w2[1]),
                   "=&v"(w2[2]), "=&v"(w2[3])
                 : "v"(code_addr), "v"(meta_addr), "i"(O2), "i"(O2 + 256), "i"(O2 + 512), "i"(O2 + 768)
                 : "memory");
  }
}

// The same for the aligned metadata (groups of 16 columns, four pieces per 2-bit unit and two per 4-bit unit): three
// dwords per piece - the one that holds its 16-bit triple word or its 4-bit group's byte, the one that holds its
// fp16 second-order scale and the one that holds its second-order zero byte - at byte 1024 + 256 q,
// 1024 + 256 (4 + q) and 1024 + 256 (8 + q) of the slot.
template <int NP>
__device__ __forceinline__ void ring_read_aligned(uint32_t code_addr, uint32_t meta_addr, uint4& q, uint32_t (&w1)[NP],
                                                  uint32_t (&w2)[NP], uint32_t (&w3)[NP]) {
  static_assert(NP == 2 || NP == 4, "pieces per unit");
  if constexpr (NP == 2) {
    asm volatile("ds_read_b128 %0, %7\n\tds_read_b32 %1, %8\n\tds_read_b32 %2, %8 offset:256\n\t"
                 "ds_read_b32 %3, %8 offset:1024\n\tds_read_b32 %4, %8 offset:1280\n\t"
                 "ds_read_b32 %5, %8 offset:2048\n\tds_read_b32 %6, %8 offset:2304\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(q), "=&v"(w1[0]), "=&v"(w1[1]), "=&v"(w2[0]), "=&v"(w2[1]), "=&v"(w3[0]), "=&v"(w3[1])
                 : "v"(code_addr), "v"(meta_addr)
                 : "memory");
  } else {
    asm volatile("ds_read_b128 %0, %13\n\tds_read_b32 %1, %14\n\tds_read_b32 %2, %14 offset:256\n\t"
                 "ds_read_b32 %3, %14 offset:512\n\tds_read_b32 %4, %14 offset:768\n\t"
                 "ds_read_b32 %5, %14 offset:1024\n\tds_read_b32 %6, %14 offset:1280\n\t"
                 "ds_read_b32 %7, %14 offset:1536\n\tds_read_b32 %8, %14 offset:1792\n\t"
                 "ds_read_b32 %9, %14 offset:2048\n\tds_read_b32 %10, %14 offset:2304\n\t"
                 "ds_read_b32 %11, %14 offset:2560\n\tds_read_b32 %12, %14 offset:2816\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(q), "=&v"(w1[0]), "=&v"(w1[1]), "=&v"(w1[2]), "=&v"(w1[3]), "=&v"(w2[0]), "=&v"(w2[1]), "=&v"(w2[2]),
                   "=&v"(w2[3]), "=&v"(w3[0]), "=&v"(w3[1]), "=&v"(w3[2]), "=&v"(w3[3])
                 : "v"(code_addr), "v"(meta_addr)
                 : "memory");
  }
}

template <int NT, int XR, int LDSB, int WV, int PU, bool AL = false>
__global__ void __launch_bounds__(WV * 64)
mpq_mms_kernel(const DevBlob b, const uint16_t* __restrict__ X, float* __restrict__ P, uint16_t* __restrict__ XT,
               const int M, const SlicePlan pl) {
#pragma clang fp contract(off)
  static_assert(WV == 8, "waves: the work split pairs wave w with wave w + 4 of the same SIMD");
  static_assert(XR == 8 || XR == 16 * NT, "staged rows");
  constexpr uint32_t W = WV, PD = 2, RMAX = 8;
  constexpr int PU4 = PU > 1 ? PU / 2 : 1;            // pieces per 2-bit unit (PU) and per 4-bit unit
  static_assert(!AL || PU == 4, "the aligned metadata comes with groups of 16 columns");
  constexpr uint32_t MW = AL ? 3 : 2;                  // dwords of scale words per lane and piece
  constexpr uint32_t SLOTB = 1024 + 256 * MW * PU;     // ring slot: codes | PU meta1 dwords per lane | PU meta2 dwords per lane (| PU more)
  constexpr uint32_t OPS = 1 + MW * PU;                // direct loads per block
  constexpr uint32_t TP = 2 / NT;  // tiles parked at a time (2 KiB per wave)
  __shared__ __align__(16) unsigned char lds[LDSB];
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t i = lane & 15u, j = lane >> 4, lane16 = lane * 16u;
  const uint32_t C = b.C, T = b.T, B2 = b.B2, B4 = C - B2;
  const uint32_t H = pl.H, NB = pl.NB, R = pl.R;
  const uint32_t h = blockIdx.x % H, band = blockIdx.x / H;
  const uint32_t a2 = h * B2 / H, n2 = (h + 1) * B2 / H - a2;   // this range's 2-bit blocks
  const uint32_t a4 = h * B4 / H, n4 = (h + 1) * B4 / H - a4;   // and 4-bit blocks
  const uint32_t len = n2 + n4;                                  // >= 1 (the host keeps H <= max(B2, B4))
  const uint32_t t0 = (uint32_t)((uint64_t)band * T / NB), ntl = (uint32_t)((uint64_t)(band + 1) * T / NB) - t0;
  const uint32_t ngroups = (ntl + R - 1) / R;                    // groups of about equal size, at most R tiles
  unsigned char* const units = lds + pl.off_units;
  float* const park0 = (float*)(lds + pl.off_park);
  unsigned char* const xbuf = lds + pl.off_xbuf;
  const DecodeConsts kc = make_consts();

  MPQ_TL_DECL
  MPQ_STAMP(0)
  // ---- once per workgroup: unit table
  dma_linear<W>(b.units, lds_addr(units), 32u * PU * C, wv, lane16);
  MPQ_VMCNT(0);
  lds_barrier();
  MPQ_STAMP(1)

  // ---- the activations of the range: every lane fills one 16-byte slot per request
  {
    const uint32_t slots2 = n2 * 4u * 8u * XR, slots = slots2 + n4 * 4u * 4u * XR;
    for (uint32_t s0 = wv * 64u; s0 < slots; s0 += W * 64u) {
      const uint32_t s = s0 + lane;
      uint32_t unit, step, m;
      if (s < slots2) {
        unit = a2 * 4u + s / (8u * XR);
        step = (s / XR) & 7u;
        m = s % XR;
      } else {
        const uint32_t s4 = s - slots2;
        unit = 4u * B2 + a4 * 4u + s4 / (4u * XR);
        step = (s4 / XR) & 3u;
        m = s4 % XR;
      }
      if (s < slots && m < (uint32_t)M) {
        // the piece (first-order group) of the unit that the step belongs to, and the step inside it
        const uint32_t spp = s < slots2 ? 8u / PU : 4u / PU4, piece = step / spp, sub = step % spp;
        const uint32_t k0x2 = *(const uint32_t*)(units + (unit * PU + piece) * 8u);
        dma16((const unsigned char*)X, m * 2u * (uint32_t)b.K + k0x2 + sub * 16u, lds_addr(xbuf) + s0 * 16u);
      }
    }
  }

  MPQ_STAMP(9)
  // ---- requests of code blocks: the enumeration (group, tile, block of the range) that the
  //      consumption below follows, restricted to every W-th block
  const uint32_t ring0 = lds_addr(lds) + wv * (PD * SLOTB);
  const uint32_t m2lane = b.off_m2 + (i >> b.m2_shift) * 4u;
  // Work split inside a group of Rn tiles: the Rn * len blocks in the order (position in the
  // range, tile) are cut into W equal pieces, one per wave.  Consecutive blocks of a wave are the
  // same position of consecutive tiles, which need the same activations: the B operands of a
  // position are read from LDS once and stay in registers for all of its tiles.
  uint32_t r_g = 0, r_s = 0, r_hi = 0, r_c = 0, r_t = 0, r_first = 0, r_Rn = 1;
#define MPQ_S_GROUP(G, FIRST, RN, LO, HI)                                               \
  {                                                                                     \
    FIRST = (G) * ntl / ngroups;                                                        \
    RN = ((G) + 1) * ntl / ngroups - FIRST;                                             \
    /* waves w and w + 4 share a SIMD and a quarter of the blocks.  The issue arbitration prefers  \
       the older wave: with equal shares it is done a quarter earlier and the SIMD runs the rest    \
       of the group with one wave (timestamps); 10/16 : 6/16 measured best (4-6 % over 8 : 8) */     \
    const uint32_t S_ = RN * len, qlo = (wv & 3u) * S_ / 4u, qhi = ((wv & 3u) + 1u) * S_ / 4u;      \
    const uint32_t mid = qlo + (qhi - qlo) * pl.older16 / 16u;                                     \
    LO = wv < 4u ? qlo : mid;                                                                      \
    HI = wv < 4u ? mid : qhi;                                                                      \
  }
#define MPQ_S_NORMALIZE                                                                 \
  while (r_g < ngroups && r_s >= r_hi) {                                                \
    if (++r_g < ngroups) {                                                              \
      MPQ_S_GROUP(r_g, r_first, r_Rn, r_s, r_hi)                                        \
      r_c = r_s / r_Rn;                                                                 \
      r_t = r_s % r_Rn;                                                                 \
    }                                                                                   \
  }
#define MPQ_S_REQUEST(SLOT)                                                             \
  {                                                                                     \
    const uint32_t blk = r_c < n2 ? a2 + r_c : B2 + a4 + (r_c - n2);                    \
    const unsigned char* tb = b.tiles + (size_t)(t0 + r_first + r_t) * b.tile_stride;   \
    const uint32_t dst = ring0 + (SLOT) * SLOTB;                                        \
    dma16(tb + b.codes_off + blk * 1024u, lane16, dst);                                 \
    /* the meta words of all PU piece slots of the lane's unit (a 4-bit unit uses the first PU4; the \
       others are padding entries that point at the zero words of the tile) */          \
    _Pragma("unroll") for (uint32_t qq = 0; qq < (uint32_t)PU; ++qq) {                  \
      const uint32_t uy = *(const uint32_t*)(units + ((blk * 4u + j) * PU + qq) * 8u + 4u); \
      if constexpr (AL) { /* Sec. 3.3 "Memory Alignment": triple word or 4-bit group's byte, second-order scale, zero byte */ \
        const uint32_t a1 = r_c < n2 ? (uy & 0xFFFCu) + i * 2u : b.off_m1b + (uy & 0xFFFFu) + i; \
        const uint32_t idx = (uy >> 16) + (i >> b.m2_shift);                            \
        dma4(tb, a1 & ~3u, dst + 1024u + qq * 256u);                                    \
        dma4(tb, (b.off_s2 + 2u * idx) & ~3u, dst + 1024u + PU * 256u + qq * 256u);     \
        dma4(tb, (b.off_z2 + idx) & ~3u, dst + 1024u + 2u * PU * 256u + qq * 256u);     \
      } else {                                                                          \
        dma4(tb, ((uy & 0xFFFFu) + i * 2u) & ~3u, dst + 1024u + qq * 256u);             \
        dma4(tb, m2lane + (uy >> 16), dst + 1024u + PU * 256u + qq * 256u);             \
      }                                                                                 \
    }                                                                                   \
    ++inflight;                                                                         \
    ++r_s;                                                                              \
    if (++r_t == r_Rn) { r_t = 0; ++r_c; }                                              \
    MPQ_S_NORMALIZE                                                                     \
  }
  if (ngroups > 0) {
    MPQ_S_GROUP(0u, r_first, r_Rn, r_s, r_hi)
    r_c = r_s / r_Rn;
    r_t = r_s % r_Rn;
  }
  uint32_t inflight = 0;
  MPQ_S_NORMALIZE
#pragma unroll
  for (uint32_t r = 0; r < PD; ++r)
    if (r_g < ngroups) MPQ_S_REQUEST(r)
  MPQ_STAMP(2)
  // the activations were requested first: they have landed when at most the block requests are left
  wait_vm((int)(OPS * inflight));
  MPQ_STAMP(3)
  lds_barrier();
  MPQ_STAMP(4)

  // ---- this workgroup's share of the transposed activations XT[k][XR] that the second kernel
  //      gathers for the outliers: the bands of a range take the range's slots in turn
  {
    const uint32_t slots2 = n2 * 4u * 8u * XR, slots = slots2 + n4 * 4u * 4u * XR;
    for (uint32_t s = band * (W * 64u) + tid; s < slots; s += NB * (W * 64u)) {
      uint32_t unit, step;
      if (s < slots2) {
        unit = a2 * 4u + s / (8u * XR);
        step = (s / XR) & 7u;
      } else {
        const uint32_t s4 = s - slots2;
        unit = 4u * B2 + a4 * 4u + s4 / (4u * XR);
        step = (s4 / XR) & 3u;
      }
      const uint32_t m = s % XR;
      if (m < (uint32_t)M) {
        const uint32_t spp = s < slots2 ? 8u / PU : 4u / PU4, piece = step / spp, sub = step % spp;
        const uint32_t k = (*(const uint32_t*)(units + (unit * PU + piece) * 8u) >> 1) + sub * 8u;
        const uint4 v = *(const uint4*)(xbuf + s * 16u);
        uint16_t* at = XT + (size_t)k * XR + m;
        at[0 * XR] = (uint16_t)v.x; at[1 * XR] = (uint16_t)(v.x >> 16);
        at[2 * XR] = (uint16_t)v.y; at[3 * XR] = (uint16_t)(v.y >> 16);
        at[4 * XR] = (uint16_t)v.z; at[5 * XR] = (uint16_t)(v.z >> 16);
        at[6 * XR] = (uint16_t)v.w; at[7 * XR] = (uint16_t)(v.w >> 16);
      }
    }
  }

  MPQ_STAMP(5)
  const uint32_t slot_lane = ring0 + lane16, meta_lane = ring0 + 1024u + lane * 4u;
  const unsigned char* xb2 = xbuf + j * (8u * XR * 16u) + (i % XR) * 16u;                        // + block * 512 * XR + step * 16 * XR
  const unsigned char* xb4 = xbuf + n2 * (512u * XR) + j * (4u * XR * 16u) + (i % XR) * 16u;      // + block * 256 * XR + step * 16 * XR
  uint32_t slot = 0;

#define MPQ_S_STEP(TWO, P, A0, A1)                                                                   \
  {                                                                                                   \
    constexpr int SPP = ((TWO) ? 8 : 4) / ((TWO) ? PU : PU4), Q = (P) / SPP;                          \
    const uint4 av = decode_step<TWO, P>(lo, hi, s1p[Q], zb[Q], kc);                                  \
    A0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                      \
                                                __builtin_bit_cast(half8_t, bx[P][0]), A0, 0, 0, 0);  \
    if (NT > 1)                                                                                       \
      A1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                    \
                                                  __builtin_bit_cast(half8_t, bx[P][NT - 1]), A1, 0, 0, 0); \
  }
// Fetch of the wave's next block: wait for it, read codes and the NP meta word pairs from its ring
// slot, refill the slot, reconstruct (s1, z1) of every piece.
#define MPQ_S_HEAD(NP, TWO)                                                                            \
  if (inflight == PD) MPQ_VMCNT(OPS * (PD - 1));                                                      \
  else MPQ_VMCNT(0); /* PD = 2: nothing else of this wave can be in flight */                         \
  uint4 q;                                                                                            \
  uint32_t w1[NP], w2[NP], w3[AL ? NP : 1];                                                           \
  if constexpr (AL) ring_read_aligned<NP>(slot_lane + slot * SLOTB, meta_lane + slot * SLOTB, q, w1, w2, w3); \
  else ring_read<NP, PU>(slot_lane + slot * SLOTB, meta_lane + slot * SLOTB, q, w1, w2);              \
  --inflight;                                                                                         \
  if (r_g < ngroups) MPQ_S_REQUEST(slot)                                                              \
  slot = slot + 1 == PD ? 0 : slot + 1;                                                               \
  half2_t s1p[NP];                                                                                    \
  half_t zb[NP];                                                                                      \
  _Pragma("unroll") for (int qq = 0; qq < NP; ++qq) {                                                 \
    if constexpr (AL) {                                                                               \
      /* the piece's table word again: where in its dwords the lane's values sit */                   \
      const uint32_t blk_ = (TWO) ? a2 + c : B2 + a4 + (c - n2);                                      \
      const uint32_t uy = *(const uint32_t*)(units + ((blk_ * 4u + j) * PU + qq) * 8u + 4u);          \
      const uint32_t idx = (uy >> 16) + (i >> b.m2_shift);                                            \
      uint32_t s_int, z1;                                                                             \
      if (TWO) {                                                                                      \
        const uint32_t w = (i & 1u) ? w1[qq] >> 16 : w1[qq] & 0xFFFFu, pos = uy & 3u;                  \
        z1 = (w >> (2u * pos)) & 3u;                                                                  \
        s_int = pos == 0 ? (w >> 6) & 15u : (w >> (pos == 1 ? 10u : 13u)) & 7u;                       \
      } else {                                                                                        \
        const uint32_t w = (w1[qq] >> (8u * ((b.off_m1b + (uy & 0xFFFFu) + i) & 3u))) & 0xFFu;        \
        s_int = w & 15u;                                                                              \
        z1 = w >> 4;                                                                                  \
      }                                                                                               \
      const uint32_t s2 = ((b.off_s2 + 2u * idx) & 2u) ? w2[qq] >> 16 : w2[qq] & 0xFFFFu;             \
      const uint32_t z2 = (w3[qq] >> (8u * ((b.off_z2 + idx) & 3u))) & 0xFFu; /* 0..15 */             \
      const half_t s1 = scale_dequant_int_zero(s_int, z2, s2);  /* exactly 0 for a padding piece */    \
      s1p[qq] = half2_t{s1, s1};                                                                      \
      zb[qq] = bits_to_half((uint16_t)(0x6400u | z1));                                                \
    } else {                                                                                          \
      const uint32_t m1 = (i & 1u) ? w1[qq] >> 16 : w1[qq] & 0xFFFFu;                                 \
      const half_t s1 = scale_dequant(m1 & 0xFFu, w2[qq]);  /* exactly 0 for a padding piece */        \
      s1p[qq] = half2_t{s1, s1};                                                                      \
      zb[qq] = bits_to_half((uint16_t)(0x6400u | (m1 >> 8)));                                         \
    }                                                                                                 \
  }                                                                                                   \
  const uint32_t lo[4] = {q.x, q.y, q.z, q.w};

  for (uint32_t g = 0; g < ngroups; ++g) {
    uint32_t first, Rn, s_at, s_hi;
    MPQ_S_GROUP(g, first, Rn, s_at, s_hi)
    float4_t acc[RMAX][2];
#pragma unroll
    for (uint32_t tt = 0; tt < RMAX; ++tt) acc[tt][0] = acc[tt][1] = float4_t{0.f, 0.f, 0.f, 0.f};
    uint32_t c = s_at / Rn, t = s_at % Rn;
    while (s_at < s_hi) {
      const uint32_t t_end = s_hi - s_at < Rn - t ? t + (s_hi - s_at) : Rn;  // tiles [t, t_end) of position c
      uint4 bx[8][NT];
      if (c < n2) {
        const unsigned char* xb0 = xb2 + c * (512u * XR);
#pragma unroll
        for (uint32_t P = 0; P < 8; ++P) {
          bx[P][0] = *(const uint4*)(xb0 + P * (16 * XR));
          if (NT > 1) bx[P][NT - 1] = *(const uint4*)(xb0 + P * (16 * XR) + 256);
        }
#pragma unroll
        for (uint32_t tt = 0; tt < RMAX; ++tt) {
          if (tt >= t && tt < t_end) {
            MPQ_S_HEAD(PU, true)
            const uint32_t hi[4] = {rotr8(q.x), rotr8(q.y), rotr8(q.z), rotr8(q.w)};
            MPQ_S_STEP(true, 0, acc[tt][0], acc[tt][1]) MPQ_S_STEP(true, 1, acc[tt][0], acc[tt][1])
            MPQ_S_STEP(true, 2, acc[tt][0], acc[tt][1]) MPQ_S_STEP(true, 3, acc[tt][0], acc[tt][1])
            MPQ_S_STEP(true, 4, acc[tt][0], acc[tt][1]) MPQ_S_STEP(true, 5, acc[tt][0], acc[tt][1])
            MPQ_S_STEP(true, 6, acc[tt][0], acc[tt][1]) MPQ_S_STEP(true, 7, acc[tt][0], acc[tt][1])
          }
        }
      } else {
        const unsigned char* xb0 = xb4 + (c - n2) * (256u * XR);
#pragma unroll
        for (uint32_t P = 0; P < 4; ++P) {
          bx[P][0] = *(const uint4*)(xb0 + P * (16 * XR));
          if (NT > 1) bx[P][NT - 1] = *(const uint4*)(xb0 + P * (16 * XR) + 256);
        }
#pragma unroll
        for (uint32_t tt = 0; tt < RMAX; ++tt) {
          if (tt >= t && tt < t_end) {
            MPQ_S_HEAD(PU4, false)
            const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
            MPQ_S_STEP(false, 0, acc[tt][0], acc[tt][1]) MPQ_S_STEP(false, 1, acc[tt][0], acc[tt][1])
            MPQ_S_STEP(false, 2, acc[tt][0], acc[tt][1]) MPQ_S_STEP(false, 3, acc[tt][0], acc[tt][1])
          }
        }
      }
      s_at += t_end - t;
      t = 0;
      ++c;
    }

    MPQ_STAMP(6)
    // ---- park the accumulators (lane l holds Y[m = l % 16 (+16)][rows 4*(l/16) .. +3] of a tile), TP
    //      tiles at a time: [wave][tile of the step][batch half][m][row]; then every output of those
    //      tiles is summed over the waves in a fixed order
#pragma unroll
    for (uint32_t st = 0; st < RMAX / TP; ++st) {
      if (st * TP >= Rn) break;
      lds_barrier();  // everybody is done reading what was parked before
      if (st == 0) { MPQ_STAMP(8) }
      float* park = park0 + wv * (TP * NT * 256u) + i * 16u + 4u * j;
      if (NT == 1) {
        *(float4_t*)(park) = acc[st * TP][0];
        *(float4_t*)(park + 256) = acc[(st * TP + 1) % RMAX][0];
      } else {
        *(float4_t*)(park) = acc[st][0];
        *(float4_t*)(park + 256) = acc[st][1];
      }
      lds_barrier();
      const uint32_t tn = Rn - st * TP < TP ? Rn - st * TP : TP;
      for (uint32_t o = tid; o < tn * NT * 256u; o += W * 64u) {
        const uint32_t m = (o >> 4) & 15u, nt = (o >> 8) % NT, tp = (o >> 8) / NT;
        const float* pk = park0 + o;  // o = ((tp * NT + nt) * 16 + m) * 16 + row inside a wave's area
        float sum = 0.f;
#pragma unroll
        for (uint32_t w2i = 0; w2i < W; ++w2i) sum += pk[w2i * (TP * NT * 256u)];
        const uint32_t tile = t0 + first + st * TP + tp;
        if (m + 16u * nt < (uint32_t)M) P[((size_t)h * T + tile) * (NT * 256u) + nt * 256u + (o & 0xFFu)] = sum;
      }
    }
  }
  MPQ_STAMP(7)
  MPQ_TL_FLUSH(blockIdx.x, wv, W - 1, lane)
#undef MPQ_S_HEAD
#undef MPQ_S_STEP
#undef MPQ_S_REQUEST
#undef MPQ_S_NORMALIZE
#undef MPQ_S_GROUP
}

// Second step of the large-batch kernel: Y[m][row] = fp16(outlier product of the row (Sec. 4.3) + the
// partial sums of the ranges, in order).  One workgroup per tile.  Outliers: 16 lanes per row, each
// takes every 16th word of the row and multiplies it with the activations of its column, which the
// first kernel left transposed (XT[k][MP]: the MP batch values of a column are one or a few 16-byte
// loads); then the lanes of a row are summed with DPP row shifts.  Batch columns >= M of XT were
// never written: their sums are computed and dropped.
template <int NT, int MP>
__global__ void __launch_bounds__(256)
mpq_mms_finish_kernel(const DevBlob b, const uint16_t* __restrict__ XT, const float* __restrict__ P,
                      uint16_t* __restrict__ Y, const int M, const int H, const uint32_t ocap) {
#pragma clang fp contract(off)
  MPQ_TL_DECL
  MPQ_STAMP(8)
  constexpr uint32_t WCAP = 2048;      // outlier words of the tile kept in LDS (the rest is read from memory)
  __shared__ float osum[MP][16];       // [batch column][row]
  __shared__ uint32_t wlds[WCAP];
  const uint32_t tile = blockIdx.x, hi4 = threadIdx.x >> 4, lo4 = threadIdx.x & 15u;
  const uint32_t* ostart = (const uint32_t*)(b.tiles + (size_t)tile * b.tile_stride + b.off_ot);
  const uint32_t* owords = ostart + MPQ_OTILE_HEAD / 4;
  // ---- everything that does not depend on another load is requested first: the row starts, the
  //      tile's words (into LDS: which row they belong to is not known yet) and the partial sums
  const uint32_t e0 = ostart[hi4], e1 = ostart[hi4 + 1];
  {
    const uint32_t nw = ocap < WCAP ? ocap : WCAP;  // the record holds ocap words (zeros after the last one)
    uint32_t wreg[WCAP / 256];
#pragma unroll
    for (uint32_t u = 0; u < WCAP / 256; ++u) wreg[u] = threadIdx.x + 256u * u < nw ? owords[threadIdx.x + 256u * u] : 0u;
#pragma unroll
    for (uint32_t u = 0; u < WCAP / 256; ++u) wlds[threadIdx.x + 256u * u] = wreg[u];
  }
  const float* p = P + (size_t)tile * (NT * 256u) + threadIdx.x;  // + nt * 256 + range * hs
  const size_t hs = (size_t)b.T * (NT * 256u);
  constexpr uint32_t PF = 6;  // partial sums requested up front (more ranges than that: the rest after the outliers)
  float pfirst[NT][PF];
#pragma unroll
  for (uint32_t nt = 0; nt < NT; ++nt) {
#pragma unroll
    for (uint32_t hh = 0; hh < PF; ++hh)
      pfirst[nt][hh] = hi4 + 16u * nt < (uint32_t)M && hh < (uint32_t)H ? p[nt * 256u + hh * hs] : 0.f;
  }
  __syncthreads();
  MPQ_STAMP(9)
  {
    const uint32_t row = hi4, q = lo4;
    float acc[MP];
#pragma unroll
    for (int m = 0; m < MP; ++m) acc[m] = 0.f;
    // four words per lane and trip, all loads issued before the first use: the chain word ->
    // activations is pure latency otherwise
    for (uint32_t e = e0 + q; e < e1; e += 64) {
      uint32_t word[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t eu = e + 16u * u;
        word[u] = eu >= e1 ? 0u : eu < WCAP ? wlds[eu] : owords[eu];
      }
      uint4 x[4][MP / 8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint4* xt = (const uint4*)(XT + (size_t)(word[u] & 0xFFFFu) * MP);
#pragma unroll
        for (int v4 = 0; v4 < MP / 8; ++v4) x[u][v4] = xt[v4];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (e + 16u * u >= e1) break;
        const float v = (float)bits_to_half((uint16_t)(word[u] >> 16));
#pragma unroll
        for (int v4 = 0; v4 < MP / 8; ++v4) {
          const uint32_t xw[4] = {x[u][v4].x, x[u][v4].y, x[u][v4].z, x[u][v4].w};
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            acc[8 * v4 + 2 * d] += v * (float)bits_to_half((uint16_t)xw[d]);
            acc[8 * v4 + 2 * d + 1] += v * (float)bits_to_half((uint16_t)(xw[d] >> 16));
          }
        }
      }
    }
#pragma unroll
    for (int m = 0; m < MP; ++m) {
      float oa = acc[m];
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x118, 0xf, 0xf, true));
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x114, 0xf, 0xf, true));
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x112, 0xf, 0xf, true));
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x111, 0xf, 0xf, true));
      if (q == 15) osum[m][row] = oa;
    }
  }
  MPQ_STAMP(10)
  __syncthreads();
  const uint32_t m = hi4, row = lo4, grow = tile * 16u + row;
#pragma unroll
  for (uint32_t nt = 0; nt < NT; ++nt) {
    const uint32_t gm = m + 16u * nt;
    if (gm >= (uint32_t)M) continue;
    float sum = osum[gm % MP][row];
#pragma unroll
    for (uint32_t hh = 0; hh < PF; ++hh)
      if (hh < (uint32_t)H) sum += pfirst[nt][hh];
    const float* pn = p + nt * 256u;
    uint32_t hh = PF;
    for (; hh + 4 <= (uint32_t)H; hh += 4) {  // four loads in flight, added in order
      const float p0 = pn[hh * hs], p1 = pn[(hh + 1) * hs], p2 = pn[(hh + 2) * hs], p3 = pn[(hh + 3) * hs];
      sum += p0; sum += p1; sum += p2; sum += p3;
    }
    for (; hh < (uint32_t)H; ++hh) sum += pn[hh * hs];
    if (grow < (uint32_t)b.N) Y[(size_t)gm * b.N + grow] = half_to_bits((half_t)sum);
  }
  MPQ_STAMP(12)
  // stamps of the second kernel: after those of 4096 workgroups of the first
  MPQ_TL_FLUSH(4096u + blockIdx.x, threadIdx.x >> 6, 3u, threadIdx.x & 63u)
}

// ------------------------------------------------------------------------------------ GEMV
//
// y = W x (Algorithm 1, the matrix-vector product at batch 1) with the outlier product of Sec. 4.3
// fused in.  Same data movement and per-block arithmetic as the batch kernel above, with everything
// batch-related folded away, and a different work split:
//
//   A workgroup of WV waves owns n consecutive 16-row tiles and treats their code blocks as ONE
//   sequence (tile 0 block 0, ..., tile 0 block C-1, tile 1 block 0, ...) that goes round-robin to
//   its waves.  A wave walks its share with a ring that stays full across tile boundaries, parks its
//   partial sums of a tile (batch column 0 of the accumulator, 16 floats) when it crosses into the
//   next tile and never waits for the other waves on the way: the workgroup meets once after the
//   staged operands have landed and once before the partial sums are added up.  The longer sequence
//   evens out the load of the waves (a tile of 19 blocks on 8 waves alone leaves five of them idle
//   for a third of the time), and the activations, the unit table and the wave's own set-up are
//   paid once per n tiles.
//
//   Outliers: groups of four waves (256 threads, 16 lanes per row) take the tiles in turn; the 16
//   lanes of a row each take every 16th word of the row and are summed with DPP row shifts.  This
//   is done right after the first barrier, while the first code blocks are still on their way, so
//   that the end of a workgroup is only: park, barrier, sum.
//
//   Order of the requests (each choice from interleaved A/B timing on one box): staged operands and
//   ONE code block per wave first; the second ring slot only after the first barrier - with every
//   request of every workgroup issued at once the memory system serves workgroup after workgroup
//   and the last ones start late.
// What the first requests of a workgroup need.  mpq_gemv_kernel takes these as its leading scalar arguments
// (14 dwords), which the loader places in registers before the first instruction: the requests go out
// without waiting for a load of the argument block (about 0.15 us per launch).
struct GemvLead {
  const unsigned char* tiles;
  const unsigned char* units;
  const uint16_t* X;
  uint32_t tile_stride, side_bytes, codes_off, C, K;
  uint32_t n_arg, n_lo, n_more;  // tiles per workgroup: at most n_arg; the first n_more workgroups n_lo + 1, the others n_lo
};

template <int PD, int LDSB, int WV, int PU, bool AL = false>
__device__ __forceinline__ void gemv_workgroup(const GemvLead& lead, const DevBlob& b, uint16_t* __restrict__ Y_arg, const uint32_t wg) {
#pragma clang fp contract(off)
  static_assert(PD >= 1 && PD <= 8 && WV >= 4 && WV <= 16, "ring depth / waves");
  __shared__ __align__(16) unsigned char lds[LDSB];
  constexpr uint32_t W = WV;
  MPQ_TL_DECL
  MPQ_STAMP(0)
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t i = lane & 15u, j = lane >> 4, lane16 = lane * 16u;
  const unsigned char* const arg_tiles = lead.tiles;
  const unsigned char* const arg_units = lead.units;
  const uint16_t* const X = lead.X;
  const uint32_t arg_stride = lead.tile_stride, arg_side = lead.side_bytes, arg_codes = lead.codes_off, arg_K = lead.K;
  const uint32_t n_arg = lead.n_arg, n_lo = lead.n_lo, n_more = lead.n_more;
  // the rest of the arguments in ONE batch of scalar loads, needed only after the first requests (the compiler
  // would fetch each field where it is first used, one dependent round trip of about 0.1 us after the other)
  uint32_t arg_m2 = b.off_m2, arg_ot = b.off_ot, arg_shift = b.m2_shift, arg_N = (uint32_t)b.N, arg_B2 = (uint32_t)b.B2;
  uint16_t* Y = Y_arg;
  const uint32_t C = lead.C;
  // The tiles are dealt evenly: the first n_more workgroups own n_lo + 1 consecutive tiles, the others n_lo
  // (n_arg = the most any of them gets).  No division here: every instruction of the prologue is paid by
  // every wave of the launch - two integer divisions at this place cost 5 % of a Llama2-7B layer.
  const uint32_t tile0 = wg * n_lo + (wg < n_more ? wg : n_more);
  const uint32_t n = n_lo + (wg < n_more ? 1u : 0u);  // tiles of this workgroup
  // LDS layout: ring | partial sums [n][W + 1][16] | side records [n] | unit table | activations
  constexpr int PU4 = PU > 1 ? PU / 2 : 1;  // pieces per 2-bit unit (PU) and per 4-bit unit
  const uint32_t units_bytes = 32u * PU * C;
  unsigned char* const ring = lds;
  float* const red = (float*)(lds + W * PD * 1024);
  unsigned char* const side0 = lds + W * PD * 1024 + (uint32_t)n_arg * (W + 1) * 64;
  unsigned char* const units = side0 + (uint32_t)n_arg * arg_side;
  unsigned char* const xs = units + units_bytes;
  const DecodeConsts kc = make_consts();

  // ---- (1) requests, oldest first: staged operands, then this wave's first code blocks
  const unsigned char* tileptr = arg_tiles + (size_t)tile0 * arg_stride;
  for (uint32_t t = 0; t < n; ++t)
    dma_linear<W>(tileptr + (size_t)t * arg_stride, lds_addr(side0) + t * arg_side, arg_side, wv, lane16);
  dma_linear<W>(arg_units, lds_addr(units), units_bytes, wv, lane16);
  dma_linear<W>((const unsigned char*)X, lds_addr(xs), 2u * arg_K, wv, lane16);
  // this wave's blocks: positions wv, wv + W, wv + 2W, ... of the n*C blocks of the workgroup
  const uint32_t ring0 = lds_addr(ring) + wv * (PD * 1024);
  const unsigned char* rbase = tileptr + arg_codes;  // code blocks of the tile being requested
  uint32_t rc = wv, rt = 0;                            // next request: block rc of tile rt (rt = n: none left)
  while (rc >= C && rt < n) { rc -= C; ++rt; rbase += arg_stride; }
  uint32_t inflight = 0;
#define MPQ_GEMV_FILL(R)                                                     \
  if (rt < n) {                                                              \
    dma16(rbase + rc * 1024u, lane16, ring0 + (R) * 1024u);                  \
    ++inflight;                                                              \
    rc += W;                                                                 \
    while (rc >= C && rt < n) { rc -= C; ++rt; rbase += arg_stride; }     \
  }
  MPQ_GEMV_FILL(0)
  asm volatile("; argument block" : "+s"(arg_m2), "+s"(arg_ot), "+s"(arg_shift), "+s"(arg_N), "+s"(arg_B2), "+s"(Y));
  MPQ_STAMP(1)
  wait_vm_upto<PD>((int)inflight);  // the staged operands have landed; the code block may still be in flight
  MPQ_STAMP(2)
  lds_barrier();
  MPQ_STAMP(3)
  // The other ring slots are requested only now.  With every request of every workgroup issued in
  // its first instructions, the memory system serves workgroup after workgroup and the last ones
  // sit idle for most of the burst; this way every workgroup gets its first block early
  // (interleaved A/B runs: 2 % on the Llama2-7B layer, 6 % on the 4096x11008 matrix).
#pragma unroll
  for (uint32_t r = 1; r < PD; ++r) MPQ_GEMV_FILL(r)
#undef MPQ_GEMV_FILL

  // ---- (2) outliers (Sec. 4.3, fused: no second kernel, no second trip to memory); all operands
  //      are already in LDS.  Four waves per tile, 16 lanes per row.  Done first, while the first
  //      code blocks are still on their way.
  {
    const uint32_t otid = tid & 255u, orow = otid >> 4, oq = otid & 15u;
    for (uint32_t t = wv >> 2; t < n && wv < (W / 4) * 4; t += W / 4) {
      const uint32_t* ostart = (const uint32_t*)(side0 + t * arg_side + arg_ot);
      const uint32_t* owords = ostart + MPQ_OTILE_HEAD / 4;
      const uint32_t rp0 = ostart[orow], rp1 = ostart[orow + 1];
      float oa = 0.f;
      for (uint32_t e = rp0 + oq; e < rp1; e += 16) {
        const uint32_t word = owords[e];
        const float v = (float)bits_to_half((uint16_t)(word >> 16));
        oa += v * (float)*(const half_t*)(xs + (word & 0xFFFFu) * 2u);
      }
      // sum over the 16 lanes of the row with DPP row shifts; lane 15 of the row ends with the total
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x118, 0xf, 0xf, true));
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x114, 0xf, 0xf, true));
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x112, 0xf, 0xf, true));
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x111, 0xf, 0xf, true));
      if (oq == 15) red[(t * (W + 1) + W) * 16 + orow] = oa;
    }
  }
  MPQ_STAMP(4)
#ifdef MPQ_TIMELINE
  uint32_t tl_blocks = 0;
#endif
  const unsigned char* unitj = units + j * (8 * PU);
  const uint32_t ringl = ring0 + lane16;
  // With three or more blocks per wave, waves in their decode steps go before waves that fetch
  // their next block (interleaved A/B runs: 4-6 % faster on the 4096x11008 and 8192x28672 shapes;
  // with fewer blocks per wave it costs 3-4 %).
  const bool decode_first = n * C >= 3u * W;
  uint32_t slot = 0;  // ring slot of the next block to consume
  uint32_t c = wv;    // next block of this wave inside the current tile (>= C: none in this tile)
  for (uint32_t t = 0; t < n; ++t) {
    const unsigned char* side = side0 + t * arg_side;
    const unsigned char* m1i = side + i * 2;
    const unsigned char* m2i = side + arg_m2 + (i >> arg_shift) * 4;
    float4_t acc0 = {0.f, 0.f, 0.f, 0.f};
#define MPQ_GEMV_STEP(TWO, P)                                                                         \
  {                                                                                                   \
    constexpr int SPP = ((TWO) ? 8 : 4) / ((TWO) ? PU : PU4), Q = (P) / SPP, PO = (P) % SPP;          \
    const uint4 av = decode_step<TWO, P>(lo, hi, s1p[Q], zb[Q], kc);                                  \
    const uint4 bv0 = *(const uint4*)(xs + xoff[Q] + 16 * PO);                                        \
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                    \
                                                  __builtin_bit_cast(half8_t, bv0), acc0, 0, 0, 0);   \
  }
#ifdef MPQ_TIMELINE
// (constant indices only: the stamps are wave-uniform and stay in scalar registers, so the timeline build
// keeps the vector register count, and with it the number of resident waves, of the product build)
#define MPQ_TL_BLOCK                                                                                    \
  {                                                                                                     \
    if (tl_blocks == 0) tl_[5] = __builtin_amdgcn_s_memrealtime();                                      \
    else if (tl_blocks == 1) tl_[6] = __builtin_amdgcn_s_memrealtime();                                 \
    else if (tl_blocks == 2) tl_[7] = __builtin_amdgcn_s_memrealtime();                                 \
    ++tl_blocks;                                                                                        \
  }
#else
#define MPQ_TL_BLOCK
#endif
#define MPQ_GEMV_BLOCK_HEAD(NP, FOUR)                                                                  \
  __builtin_amdgcn_s_setprio(0);                                                                      \
  /* the block's unit table entries are requested first: the wait inside the ring read below covers  \
     them, so the scale words can be requested right after it */                                     \
  uint2 ent[NP];                                                                                      \
  _Pragma("unroll") for (int qq = 0; qq < NP; ++qq) ent[qq] = *(const uint2*)(unitj + c * (32u * PU) + 8 * qq); \
  /* requests younger than the block needed now: the other blocks in flight (the run-time switch of  \
     wait_vm is kept out of the two-slot ring: its compare chain sat on the tail of every workgroup) */ \
  if (inflight == PD) MPQ_VMCNT(PD - 1); else if (PD == 2) MPQ_VMCNT(0); else wait_vm((int)inflight - 1); \
  uint4 q;                                                                                            \
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(q) : "v"(ringl + slot * 1024u) : "memory"); \
  --inflight;                                                                                         \
  if (rt < n) { /* refill the freed slot with the next block of this wave's sequence */               \
    dma16(rbase + rc * 1024u, lane16, ring0 + slot * 1024u);                                          \
    ++inflight;                                                                                       \
    rc += W;                                                                                          \
    while (rc >= C && rt < n) { rc -= C; ++rt; rbase += arg_stride; }                              \
  }                                                                                                   \
  slot = slot + 1 == PD ? 0 : slot + 1;                                                               \
  half2_t s1p[NP];                                                                                    \
  half_t zb[NP];                                                                                      \
  uint32_t xoff[NP];                                                                                  \
  if constexpr (AL) pieces_aligned<NP, FOUR>(ent, side, b, i, s1p, zb, xoff);                         \
  else finish_pieces<NP>(ent, m1i, m2i, s1p, zb, xoff);                                               \
  if (decode_first) __builtin_amdgcn_s_setprio(2);                                                    \
  MPQ_TL_BLOCK                                                                                        \
  const uint32_t lo[4] = {q.x, q.y, q.z, q.w};
    for (; c < arg_B2; c += W) {
      MPQ_GEMV_BLOCK_HEAD(PU, false)
      const uint32_t hi[4] = {rotr8(q.x), rotr8(q.y), rotr8(q.z), rotr8(q.w)};
      MPQ_GEMV_STEP(true, 0) MPQ_GEMV_STEP(true, 1) MPQ_GEMV_STEP(true, 2) MPQ_GEMV_STEP(true, 3)
      MPQ_GEMV_STEP(true, 4) MPQ_GEMV_STEP(true, 5) MPQ_GEMV_STEP(true, 6) MPQ_GEMV_STEP(true, 7)
    }
    for (; c < C; c += W) {
      MPQ_GEMV_BLOCK_HEAD(PU4, true)
      const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
      MPQ_GEMV_STEP(false, 0) MPQ_GEMV_STEP(false, 1) MPQ_GEMV_STEP(false, 2) MPQ_GEMV_STEP(false, 3)
    }
#undef MPQ_GEMV_BLOCK_HEAD
#undef MPQ_GEMV_STEP
    __builtin_amdgcn_s_setprio(0);
    c -= C;  // the sequence continues in the next tile
    // accumulator lane l holds Y[m = l % 16][rows 4*(l/16) .. +3]; only batch column 0 is real
    if (i == 0) *(float4_t*)(red + (t * (W + 1) + wv) * 16 + 4 * j) = acc0;
  }

  MPQ_STAMP(8)
  lds_barrier();
  MPQ_STAMP(9)
  // ---- (3) row r of tile t: the outlier term and the W partial sums, in a fixed order
  if (tid < 16 * n) {
    const uint32_t t = tid >> 4, r = tid & 15u;
    const float* rt0 = red + t * (W + 1) * 16 + r;
    float sum = rt0[W * 16];
#pragma unroll
    for (uint32_t w2 = 0; w2 < W; ++w2) sum += rt0[w2 * 16];
    const uint32_t row = (tile0 + t) * 16 + r;
    if (row < arg_N) Y[row] = half_to_bits((half_t)sum);
  }
  MPQ_STAMP(10)
#ifdef MPQ_TIMELINE
  MPQ_TL_NOTE(11, tl_blocks)
#endif
  MPQ_TL_FLUSH(wg, wv, W - 1, lane)
}

template <int PD, int LDSB, int WV, int PU = 1, bool AL = false>
__global__ void __launch_bounds__(WV * 64)
mpq_gemv_kernel(const unsigned char* __restrict__ tiles, const unsigned char* __restrict__ units, const uint16_t* __restrict__ X,
                const uint32_t tile_stride, const uint32_t side_bytes, const uint32_t codes_off, const uint32_t C, const uint32_t K,
                const uint32_t n_arg, const uint32_t n_lo, const uint32_t n_more, const DevBlob b, uint16_t* __restrict__ Y) {
  const GemvLead lead = {tiles, units, X, tile_stride, side_bytes, codes_off, C, K, n_arg, n_lo, n_more};
  gemv_workgroup<PD, LDSB, WV, PU, AL>(lead, b, Y, blockIdx.x);
}

// Several independent matrix-vector products in one launch (separate projections of a layer, the
// experts a token is routed to): workgroups [first[p], first[p + 1]) work on problem p, one tile
// each.  Saves the fixed cost of a launch (about 2.5 us here) per product after the first.
struct MultiArgs {
  DevBlob b[MPQ_MAX_MULTI];
  const uint16_t* X[MPQ_MAX_MULTI];
  uint16_t* Y[MPQ_MAX_MULTI];
  uint32_t first[MPQ_MAX_MULTI + 1];
  int32_t count;
};

template <int PD, int LDSB, int WV, int PU = 1, bool AL = false>
__global__ void __launch_bounds__(WV * 64)
mpq_gemv_multi_kernel(const MultiArgs a) {
  uint32_t p = 0;
  while ((int32_t)p + 1 < a.count && blockIdx.x >= a.first[p + 1]) ++p;
  const DevBlob b = a.b[p];
  const GemvLead lead = {b.tiles, b.units, a.X[p], b.tile_stride, b.side_bytes, b.codes_off, (uint32_t)b.C, (uint32_t)b.K, 1u, 1u, 0u};
  gemv_workgroup<PD, LDSB, WV, PU, AL>(lead, b, a.Y[p], blockIdx.x - a.first[p]);
}

// ------------------------------------------------------------------------------------ GEMV, plane sums
//
// y = W x at batch 1 (Algorithm 1 + Sec. 4.3) with the 2-bit groups evaluated WITHOUT decoding a
// single weight, bit-identical in its use of the per-weight fp16 rounding of eq. 5:
//
//   A 2-bit code c of (row, group) decodes to one of four fp16 numbers T[c] = fp16((c - z1) * s1).
//   With b0, b1 the bits of c and g(c) = {0, 1, 2, 4}[c] = b0 + 2 b1 + b0 b1,
//       T[c] = T0 + (T1 - T0) b0 + (T2 - T0) b1 + (T3 - T2 - T1 + T0) b0 b1,
//   so the group's part of the row sum is
//       T0 A + (e1 - d) S0 + (e2 / 2 - d) S1 + d Sg,   e1 = T1 - T0, e2 = T2 - T0, d = T3 - T2 - e1,
//       A = sum x_k,  S0 = sum b0 x_k,  S1 = sum 2 b1 x_k,  Sg = sum g(c_k) x_k   over the group's columns.
//   The four T are computed exactly as the definition rounds them; only the order of the fp32
//   additions differs from a per-weight loop.
//
//   S0, S1, Sg come from v_mfma_scale_f32_16x16x128_f8f6f4.  Its B operand is fp4 (E2M1): the blob
//   keeps the two bits of a code in the two exponent bits of a nibble (mpq_format.h), so
//   dword & 0x22222222 / 0x44444444 / 0x66666666 are eight fp4 numbers b0 / 2 b1 / g(c) each - three
//   vector instructions per 8 weights and plane, none per weight.  Lane (j, i) of a block holds unit j
//   of row i = 32 nibbles = the instruction's contraction slots 32 j .. 32 j + 31 of column i; the
//   last 32 columns of the unit are the same nibbles of the dword rotated right by 2.
//   Its A operand is fp8 (E4M3): the activations, split once per workgroup into three pieces
//   x = p0 + p1 + p2 (each the fp8 rounding of what the previous ones left: 12 significant bits, exact
//   for fp16 inputs), scaled per 64-column unit by a power of two that the instruction's per-block
//   scale operand undoes.  Row 4 g + p of A holds piece p of unit g on the slots of unit g and zeros
//   elsewhere, so D[4 g + p][i] = sum over unit g of piece p times plane: lane (j, i) of the result
//   holds, in its four registers, the three piece sums of ITS unit and row.  The instruction adds
//   products in a window of about 14 bits below the largest product of a dot product before the
//   fp32 accumulate; every piece has 4 significant bits, so columns within 2^-10 of the largest of
//   their 32-column half unit are exact.  Activations must be finite.
//
//   4-bit groups have 16 values per (row, group); they take the per-weight decode and the f16 matrix
//   instruction as in the other kernels.
//
// Data movement.  No request of a wave depends on data another request brings: code blocks and the
// (s_int, z1), (s2, z2) words of their lanes travel together into a per-wave ring (three direct
// global->LDS loads per block; the addresses of a wave's first requests come from the kernel arguments), so a wave
// issues its first blocks in its first instructions.  A workgroup of WV waves owns n consecutive
// tiles and treats their blocks as one sequence dealt round-robin to its waves; the activations are
// staged and split once per workgroup while the first blocks are in flight.  Outliers of tile t are
// summed by wave t from a record the wave fetched for itself.  Three barriers per workgroup.
struct PlanePlan {
  uint32_t off_park, off_units, off_xs, off_utab, off_pieces, off_zero, off_obuf;  // LDS byte offsets (ring at 0)
  uint32_t obuf_bytes;  // outlier record of a tile: 128 + 4 * ocap
  uint32_t n;           // tiles per workgroup (<= WV)
  uint32_t x_lds;       // 1: the whole activation vector is staged at off_xs; 0 (rows too long for that): only the
                        //    columns of the 4-bit units are copied there (64 bytes per unit), the split and the
                        //    outliers read the activations from memory
  // Dealing of the workgroup's blocks: wave w takes the run [N cum[w] / cum[W], N cum[w + 1] / cum[W]) of
  // its N blocks.  Older waves (lower numbers; waves w, w + 4, ... share a SIMD) win the issue arbitration
  // and run faster; they get longer runs so that all waves end together.
  uint32_t cum[17];
};
#define MPQ_PLANE_MAX_UNITS 512
struct PlaneArgs {
  DevBlob b;
  const uint16_t* X;
  uint16_t* Y;
  PlanePlan pl;
  // word 1 (meta1 offset | meta2 offset << 16) of every unit's table entry, rebuilt on the host from the
  // header: the first requests of a wave take their addresses from here, i.e. from the kernel arguments
  // every wave loads anyway, and depend on no other load
  uint32_t uw[MPQ_PLANE_MAX_UNITS];
};

typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef short short2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float quad_add(float v) {  // sum over the 4 lanes of a quad, all lanes get it
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));  // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));  // quad_perm [2,3,0,1]
  return v;
}
__device__ __forceinline__ uint32_t quad_max(uint32_t v) {
  uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xf, 0xf, true);
  v = v > o ? v : o;
  o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xf, 0xf, true);
  return v > o ? v : o;
}

// Reads ring slot contents and one more LDS dword in one go: the 16 bytes of codes of the lane, its
// (s_int, z1) and (s2, z2) dwords, and the unit word at `uaddr` that the next request needs.  One asm
// statement with its wait: nothing may be scheduled between a read and the wait.
__device__ __forceinline__ void plane_ring_read(uint32_t code_addr, uint32_t meta_addr, uint32_t uaddr, uint4& q, uint32_t& w1,
                                                uint32_t& w2, uint32_t& uy) {
  asm volatile("ds_read_b128 %0, %4\n\tds_read_b32 %1, %5\n\tds_read_b32 %2, %5 offset:256\n\tds_read_b32 %3, %6 offset:4\n\t"
               "s_waitcnt lgkmcnt(0)"
               : "=&v"(q), "=&v"(w1), "=&v"(w2), "=&v"(uy)
               : "v"(code_addr), "v"(meta_addr), "v"(uaddr)
               : "memory");
}

template <int LDSB, int WV>
__global__ void __launch_bounds__(WV * 64)
mpq_gemvp_kernel(const PlaneArgs a) {
#pragma clang fp contract(off)
  // Two ring slots per wave.  The wave keeps exactly two blocks in flight from its first request to its
  // last fetch - past the end of its run it re-requests its last block - so that "the block I need has
  // landed" is the same wait everywhere (vmcnt(3): the three requests of the other slot) and the loop
  // carries no counters for it.  Scalar instructions cost issue slots like vector ones: the loop is
  // written to need few of either.
  constexpr uint32_t W = WV, SLOTB = 1536;
  __shared__ __align__(16) unsigned char lds[LDSB];
  MPQ_TL_DECL
  MPQ_STAMP(0)
  const DevBlob& b = a.b;
  const PlanePlan& pl = a.pl;
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t i = lane & 15u, j = lane >> 4, lane16 = lane * 16u;
  const uint32_t C = b.C, T = b.T, B2 = b.B2;
  const uint32_t tile0 = blockIdx.x * pl.n;
  const uint32_t n = T - tile0 < pl.n ? T - tile0 : pl.n;
  float* const red = (float*)(lds + pl.off_park);  // [n][2 W + 1][16]
  unsigned char* const units = lds + pl.off_units;
  unsigned char* const xs = lds + pl.off_xs;
  unsigned char* const utab = lds + pl.off_utab;
  unsigned char* const pieces = lds + pl.off_pieces;
  const DecodeConsts kc = make_consts();

  // ---- (1) requests: the staged operands (activations first: everything waits for them), then the
  //      wave's first two blocks, whose unit words come from the kernel arguments
  const unsigned char* tileptr = b.tiles + (size_t)tile0 * b.tile_stride;
  const unsigned char* const xg = (const unsigned char*)a.X;
  const bool x_lds = pl.x_lds != 0;
  if (x_lds) dma_linear<W>(xg, lds_addr(xs), 2u * b.K, wv, lane16);
  dma_linear<W>(b.units, lds_addr(units), 32u * C, wv, lane16);
  // outliers of tile t: waves og * t .. og * t + og - 1 counted from the last wave down (the first waves
  // have the activations to split); the first wave of a group fetches the tile's record
  const uint32_t og = 4u * n <= W ? 4u : 1u;          // waves per tile: 16 or 4 lanes per row
  const uint32_t ow = W - 1u - wv, ot = ow / og;      // this wave works on the outliers of tile ot (if < n)
  if (ot < n && ow % og == 0) {
    const unsigned char* rec = tileptr + (size_t)ot * b.tile_stride + b.off_ot;
    const uint32_t dst = lds_addr(lds + pl.off_obuf) + ot * pl.obuf_bytes;
    for (uint32_t off = 0; off < pl.obuf_bytes; off += 1024u)
      if (off + lane16 < pl.obuf_bytes) dma16(rec + off, lane16, dst + off);
  }
  // this wave's blocks: the contiguous run [k0, k1) of the workgroup's n C blocks (tile after tile, the
  // 2-bit blocks of a tile before its 4-bit blocks); the runs of older waves are longer (see PlanePlan)
  const uint32_t nblk = n * C;
  const uint32_t k0 = nblk * pl.cum[wv] / pl.cum[W], k1 = nblk * pl.cum[wv + 1] / pl.cum[W];
  const uint32_t t_first = k0 / C, c_first = k0 - t_first * C;
  const uint32_t ring0 = lds_addr(lds) + wv * (2u * SLOTB);
  const uint32_t m1l = (i * 2u) & ~3u;  // inside a group's 32 bytes of (s_int, z1) pairs: the dword with this row's pair
  const uint32_t m2lane = b.off_m2 + (i >> b.m2_shift) * 4u;
  const unsigned char* rtile = tileptr + (size_t)t_first * b.tile_stride;  // record of the tile being requested
  const unsigned char* rcode = rtile + b.codes_off + c_first * 1024u;      // its block requested next
  uint32_t rc = c_first, rleft = k1 > k0 ? k1 - k0 - 1u : 0u;  // that block's number; blocks after it in the run
  uint32_t rdst = ring0;                                        // ring slot the next request fills
  uint32_t uaddr = pl.off_units + j * 8u + c_first * 32u;        // LDS address of the unit entry of lane (j, .) of block rc
// one block: codes, then the lane's (s_int, z1) dword and (s2, z2) dword (group offsets are multiples of 32)
#define MPQ_P_REQUEST(UY)                                                              \
  {                                                                                    \
    const uint32_t uy = (UY);                                                          \
    dma16(rcode, lane16, rdst);                                                        \
    dma4(rtile, (uy & 0xFFFFu) | m1l, rdst + 1024u);                                   \
    dma4(rtile, m2lane + (uy >> 16), rdst + 1280u);                                    \
    rdst = 2u * ring0 + SLOTB - rdst; /* the other slot */                             \
    if (rleft > 0) { /* past the end of the run the last block is requested again */   \
      --rleft;                                                                         \
      rcode += 1024;                                                                   \
      uaddr += 32u;                                                                    \
      if (++rc == C) {                                                                 \
        rc = 0;                                                                        \
        rtile += b.tile_stride;                                                        \
        rcode = rtile + b.codes_off;                                                   \
        uaddr = pl.off_units + j * 8u;                                                 \
      }                                                                                \
    }                                                                                  \
  }
  if (k1 > k0) {
    // unit words of the first two blocks by scalar loads from the kernel arguments (the table has not
    // landed in LDS yet); written out: a vector load here would count against the vmcnt waits
    typedef uint32_t u4_s __attribute__((ext_vector_type(4)));
    const unsigned char* kuw = (const unsigned char*)(uintptr_t)__builtin_amdgcn_kernarg_segment_ptr() + offsetof(PlaneArgs, uw);
    const uint32_t c_second = rleft > 0 ? (c_first + 1u == C ? 0u : c_first + 1u) : c_first;
    u4_s u0, u1;
    asm volatile("s_load_dwordx4 %0, %2, %3\n\ts_load_dwordx4 %1, %2, %4\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(u0), "=&s"(u1)
                 : "s"(kuw), "s"(__builtin_amdgcn_readfirstlane(c_first) * 16u), "s"(__builtin_amdgcn_readfirstlane(c_second) * 16u)
                 : "memory");
    MPQ_P_REQUEST(j == 0 ? u0[0] : j == 1 ? u0[1] : j == 2 ? u0[2] : u0[3])
    MPQ_P_REQUEST(j == 0 ? u1[0] : j == 1 ? u1[1] : j == 2 ? u1[2] : u1[3])
  }
  MPQ_STAMP(1)
  if (tid < 32) ((uint32_t*)(lds + pl.off_zero))[tid] = 0u;  // what inactive lanes of the A operand read
  for (uint32_t o = tid; o < n * (2u * W + 1u) * 16u; o += W * 64u) red[o] = 0.f;  // a wave parks sums only for the tiles it touches
  if (k1 > k0) MPQ_VMCNT(6); else MPQ_VMCNT(0);  // what is older than the two blocks has landed: activations, unit table, outlier record
  MPQ_STAMP(2)
  lds_barrier();
  MPQ_STAMP(3)

  // ---- (2) split the activations of every 2-bit unit into three fp8 pieces, in the order of the
  //      instruction's contraction slots.  16 lanes per unit: lane (pass, d, hf) takes the two dwords of
  //      activations that hold the columns of nibbles 2 hf, 2 hf + 1 (low halves) and 2 hf + 4, 2 hf + 5
  //      (high halves) of dword d of the codes, for the first (pass 0) or last 32 columns of the unit.
  {
    const uint32_t items = 64u * B2;
    for (uint32_t it = tid; it < items; it += W * 64u) {
      const uint32_t u = it >> 4, pass = (it >> 3) & 1u, d = (it >> 1) & 3u, hf = it & 1u;
      const uint2 ue = *(const uint2*)(units + u * 8u);
      const bool real = (ue.y & 0xFFFFu) != 32u * (uint32_t)b.G;  // padding units point at the zero entries
      // slot 8 d + nn of the half unit <-> column 8 (nn % 4) + 2 d + nn / 4
      const uint32_t xat = ue.x + 64u * pass + 32u * hf + 4u * d;
      uint32_t x0 = 0u, x1 = 0u;
      if (real) {
        if (x_lds) { x0 = *(const uint32_t*)(xs + xat); x1 = *(const uint32_t*)(xs + xat + 16u); }
        else { x0 = *(const uint32_t*)(xg + xat); x1 = *(const uint32_t*)(xg + xat + 16u); }  // ordinary loads: waited for in full
      }
      float sum = ((float)as_h2(x0).x + (float)as_h2(x0).y) + ((float)as_h2(x1).x + (float)as_h2(x1).y);
      typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
      const ushort2_t m2 = __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, x0 & 0x7FFF7FFFu), __builtin_bit_cast(ushort2_t, x1 & 0x7FFF7FFFu));
      uint32_t mx = m2.x > m2.y ? m2.x : m2.y;   // bit pattern of the largest magnitude of the item
      // sum and largest magnitude of the unit: over its 16 lanes (a row of the wave), every lane gets them
      sum = quad_add(sum);
      mx = quad_max(mx);
      sum += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, sum), 0x141, 0xf, 0xf, true));  // row_half_mirror
      sum += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, sum), 0x140, 0xf, 0xf, true));  // row_mirror
      {
        uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)mx, 0x141, 0xf, 0xf, true);
        mx = mx > o ? mx : o;
        o = (uint32_t)__builtin_amdgcn_mov_dpp((int)mx, 0x140, 0xf, 0xf, true);
        mx = mx > o ? mx : o;
      }
      uint32_t E = mx >> 10;  // exponent field of the largest magnitude of the unit
      E = E < 1u ? 1u : E > 30u ? 30u : E;
      // x' = x * 2^(15 - E): the largest is in [1, 2); pieces are fp8(x' 2^7), fp8(rest 2^11), fp8(rest 2^15)
      const uint32_t mbits = E < 30u ? (30u - E) << 10 : 0x0200u;
      const half2_t mult = as_h2(mbits | (mbits << 16));
      short2_t q0 = {0, 0}, q1 = {0, 0}, q2 = {0, 0};  // bytes: pair 0 low, pair 0 high, pair 1 low, pair 1 high
      // ENC(v, s) = fp8(v / s) of both halves of v into the low or high word; DEC(p, s) = p * s
#define MPQ_P_SPLIT(XV, HI)                                                                           \
  {                                                                                                   \
    const half2_t xm = as_h2(XV) * mult;                                                              \
    q0 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(q0, xm, 0.0078125f, HI);                            \
    half2_t dc = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(__builtin_bit_cast(int, q0), 0.0078125f, HI); \
    half2_t r = xm - dc;                                                                              \
    q1 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(q1, r, 0.00048828125f, HI);                         \
    dc = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(__builtin_bit_cast(int, q1), 0.00048828125f, HI);   \
    r = r - dc;                                                                                       \
    q2 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(q2, r, 0.000030517578125f, HI);                     \
  }
      MPQ_P_SPLIT(x0, false)
      MPQ_P_SPLIT(x1, true)
#undef MPQ_P_SPLIT
      // slots 8 d + 2 hf, + 1 take the low halves of the two pairs, slots 8 d + 4 + 2 hf, + 1 their high halves
      unsigned char* pd = pieces + u * 192u + pass * 96u + d * 8u + hf * 2u;
      const uint32_t p0 = (uint32_t)__builtin_bit_cast(int, q0), p1 = (uint32_t)__builtin_bit_cast(int, q1), p2 = (uint32_t)__builtin_bit_cast(int, q2);
      *(uint16_t*)(pd) = (uint16_t)__builtin_amdgcn_perm(0u, p0, 0x0c0c0200u);
      *(uint16_t*)(pd + 4u) = (uint16_t)__builtin_amdgcn_perm(0u, p0, 0x0c0c0301u);
      *(uint16_t*)(pd + 32u) = (uint16_t)__builtin_amdgcn_perm(0u, p1, 0x0c0c0200u);
      *(uint16_t*)(pd + 36u) = (uint16_t)__builtin_amdgcn_perm(0u, p1, 0x0c0c0301u);
      *(uint16_t*)(pd + 64u) = (uint16_t)__builtin_amdgcn_perm(0u, p2, 0x0c0c0200u);
      *(uint16_t*)(pd + 68u) = (uint16_t)__builtin_amdgcn_perm(0u, p2, 0x0c0c0301u);
      // per unit: the sum of its activations and the exponent byte of piece 0's scale, 2^(E - 22)
      if ((it & 15u) == 0) *(uint2*)(utab + u * 8u) = uint2{__builtin_bit_cast(uint32_t, sum), 105u + E};
    }
    if (!x_lds) {
      // the activations of the 4-bit units (32 columns = 64 bytes each), where the 4-bit blocks will look for them
      for (uint32_t it = tid; it < 16u * (C - B2); it += W * 64u) {
        const uint32_t u4 = it >> 2, part = it & 3u;
        const uint32_t k0x2 = *(const uint32_t*)(units + (4u * B2 + u4) * 8u);
        *(uint4*)(xs + u4 * 64u + part * 16u) = *(const uint4*)(xg + k0x2 + part * 16u);
      }
    }
  }

  MPQ_STAMP(4)
  // ---- (3) outliers (Sec. 4.3, fused): og waves per tile, 64 og / 16 lanes per row, two words per
  //      lane in flight
  if (ot < n) {
    const uint32_t* ostart = (const uint32_t*)(lds + pl.off_obuf + ot * pl.obuf_bytes);
    const uint32_t* owords = ostart + MPQ_OTILE_HEAD / 4;
    const uint32_t lpr = 4u * og;                              // lanes per row
    const uint32_t ol = (ow % og) * 64u + lane;                // lane index inside the tile's group of waves
    const uint32_t orow = ol / lpr, oq = ol % lpr;
    const uint32_t rp0 = ostart[orow], rp1 = ostart[orow + 1];
    float oa = 0.f, ob = 0.f;
    for (uint32_t e = rp0 + oq; e < rp1; e += 2u * lpr) {
      const uint32_t wa = owords[e], wb = e + lpr < rp1 ? owords[e + lpr] : 0u;
      const unsigned char* xo = x_lds ? xs : xg;
      const float xa = (float)*(const half_t*)(xo + (wa & 0xFFFFu) * 2u), xb = (float)*(const half_t*)(xo + (wb & 0xFFFFu) * 2u);
      oa = __builtin_fmaf((float)bits_to_half((uint16_t)(wa >> 16)), xa, oa);
      ob = __builtin_fmaf((float)bits_to_half((uint16_t)(wb >> 16)), xb, ob);
    }
    oa += ob;
    oa = quad_add(oa);
    if (og == 4u) {  // 16 lanes per row: lane 15 of the row ends with the total
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x114, 0xf, 0xf, true));
      oa += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, oa), 0x118, 0xf, 0xf, true));
      if (oq == 15u) red[(ot * (2 * W + 1) + 2 * W) * 16 + orow] = oa;
    } else if (oq == 0u) {
      red[(ot * (2 * W + 1) + 2 * W) * 16 + orow] = oa;
    }
  }
  MPQ_STAMP(5)
  lds_barrier();
  MPQ_STAMP(6)

  // ---- (4) this wave's blocks, in order
  // A operand of lane (j, m = 4 g + p): piece p of unit g of the block on the 16 slots this lane
  // covers (low 16 bytes: slots 16 j .. 16 j + 15, high 16 bytes: slots 64 + 16 j ..), zeros elsewhere
  const uint32_t ga = i >> 2, pa = i & 3u;
  const bool act = (j >> 1) == (ga & 1u) && pa < 3u;
  const uint32_t chunk = pl.off_pieces + ga * 192u + pa * 32u + (j & 1u) * 16u;
  const uint32_t a_lo0 = act && ga < 2u ? chunk : pl.off_zero, a_lo1 = act && ga < 2u ? 768u : 0u;
  const uint32_t a_hi0 = act && ga >= 2u ? chunk : pl.off_zero, a_hi1 = act && ga >= 2u ? 768u : 0u;
  const int sc_lane = -4 * (int)pa;
  const uint32_t unit_lane = pl.off_units + j * 8u, utab_lane = pl.off_utab + j * 8u;
  uint32_t code_addr = ring0 + lane16, meta_addr = ring0 + 1024u + lane * 4u;  // of the slot read next
  float one;
  asm volatile("v_mov_b32 %0, 1.0" : "=v"(one));  // opaque to the optimiser: keeps x * one - y a single fma
  {
    uint32_t t = t_first, c = c_first;       // the wave's current block: block c of tile t
    float yacc = 0.f;                        // row i, units j of this wave's 2-bit blocks of the tile
    float4_t acc4 = {0.f, 0.f, 0.f, 0.f};    // its 4-bit blocks (batch column 0 of the f16 instruction)
    for (uint32_t todo = k1 - k0; todo > 0; --todo) {
      MPQ_VMCNT(3);  // the block has landed: only the three requests of the other slot are younger
      uint4 q;
      uint32_t w1, w2, unit_word;
      plane_ring_read(code_addr, meta_addr, uaddr, q, w1, w2, unit_word);
      MPQ_P_REQUEST(unit_word)
      code_addr = 2u * (ring0 + lane16) + SLOTB - code_addr;
      meta_addr = 2u * (ring0 + 1024u + lane * 4u) + SLOTB - meta_addr;
      // (s1, z1) of the lane's (row, unit) from the scale words that came with the block
      const uint32_t m1 = (i & 1u) ? w1 >> 16 : w1 & 0xFFFFu;
      const half_t s1 = scale_dequant(m1 & 0xFFu, w2);  // exactly 0 for a padding unit
      const half2_t s1p = {s1, s1};
      const half_t zb = bits_to_half((uint16_t)(0x6400u | (m1 >> 8)));  // 1024 + z1
      if (c < B2) {
        const uint2 ut = *(const uint2*)(lds + utab_lane + c * 32u);
        const uint32_t alo = __umul24(c, a_lo1) + a_lo0, ahi = __umul24(c, a_hi1) + a_hi0;
        const uint4 ax0 = *(const uint4*)(lds + alo), ax1 = *(const uint4*)(lds + ahi);
        const uint4 ay0 = *(const uint4*)(lds + alo + 96u), ay1 = *(const uint4*)(lds + ahi + 96u);
        const int sca = (int)ut.y + sc_lane;
        const v8i_t ax = {(int)ax0.x, (int)ax0.y, (int)ax0.z, (int)ax0.w, (int)ax1.x, (int)ax1.y, (int)ax1.z, (int)ax1.w};
        const v8i_t ay = {(int)ay0.x, (int)ay0.y, (int)ay0.z, (int)ay0.w, (int)ay1.x, (int)ay1.y, (int)ay1.z, (int)ay1.w};
        const uint32_t r0 = __builtin_amdgcn_alignbit(q.x, q.x, 2), r1 = __builtin_amdgcn_alignbit(q.y, q.y, 2);
        const uint32_t r2 = __builtin_amdgcn_alignbit(q.z, q.z, 2), r3 = __builtin_amdgcn_alignbit(q.w, q.w, 2);
#define MPQ_P_PLANE(MASK, X0, X1, X2, X3) \
  v8i_t{(int)((X0) & (MASK)), (int)((X1) & (MASK)), (int)((X2) & (MASK)), (int)((X3) & (MASK)), 0, 0, 0, 0}
#define MPQ_P_MFMA(A, B, ACC) __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B, ACC, 0, 4, 0, sca, 0, 0x7F7F7F7F)
        const float4_t z4 = {0.f, 0.f, 0.f, 0.f};
        float4_t s0 = MPQ_P_MFMA(ax, MPQ_P_PLANE(0x22222222u, q.x, q.y, q.z, q.w), z4);
        float4_t sb = MPQ_P_MFMA(ax, MPQ_P_PLANE(0x44444444u, q.x, q.y, q.z, q.w), z4);
        float4_t sg = MPQ_P_MFMA(ax, MPQ_P_PLANE(0x66666666u, q.x, q.y, q.z, q.w), z4);
        s0 = MPQ_P_MFMA(ay, MPQ_P_PLANE(0x22222222u, r0, r1, r2, r3), s0);
        sb = MPQ_P_MFMA(ay, MPQ_P_PLANE(0x44444444u, r0, r1, r2, r3), sb);
        sg = MPQ_P_MFMA(ay, MPQ_P_PLANE(0x66666666u, r0, r1, r2, r3), sg);
#undef MPQ_P_MFMA
#undef MPQ_P_PLANE
        // the four values a code of this (row, unit) decodes to, rounded as eq. 5 rounds them
        const half2_t zbp = {zb, zb};
        const half2_t t01 = (half2_t{(half_t)1024.f, (half_t)1025.f} - zbp) * s1p;
        const half2_t t23 = (half2_t{(half_t)1026.f, (half_t)1027.f} - zbp) * s1p;
        // differences of halves as mixed-precision fmas (x * one - y): one instruction each
        const float T0 = (float)t01.x;
        const float e1 = __builtin_fmaf((float)t01.y, one, -T0), e2 = __builtin_fmaf((float)t23.x, one, -T0);
        const float dl = __builtin_fmaf((float)t23.y, one, -(float)t23.x) - e1;
        const float c0 = e1 - dl, c1 = __builtin_fmaf(0.5f, e2, -dl);
        yacc = __builtin_fmaf(T0, __builtin_bit_cast(float, ut.x), yacc);
        const float S0 = (s0[0] + s0[1]) + s0[2], S1 = (sb[0] + sb[1]) + sb[2], Sg = (sg[0] + sg[1]) + sg[2];
        yacc = __builtin_fmaf(c0, S0, yacc);
        yacc = __builtin_fmaf(c1, S1, yacc);
        yacc = __builtin_fmaf(dl, Sg, yacc);
      } else {
        // a 4-bit block: every weight decoded (eq. 5), the f16 matrix instruction multiplies and adds
        const uint32_t xoff = x_lds ? *(const uint32_t*)(lds + unit_lane + c * 32u) : (4u * (c - B2) + j) * 64u;
        const uint32_t lo[4] = {q.x, q.y, q.z, q.w};
        const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
#define MPQ_P_STEP4(P)                                                                                \
  {                                                                                                   \
    const uint4 av = decode_step<false, P>(lo, hi, s1p, zb, kc);                                      \
    const uint4 bv = *(const uint4*)(xs + xoff + 16 * (P));                                           \
    acc4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),                    \
                                                  __builtin_bit_cast(half8_t, bv), acc4, 0, 0, 0);    \
  }
        MPQ_P_STEP4(0) MPQ_P_STEP4(1) MPQ_P_STEP4(2) MPQ_P_STEP4(3)
#undef MPQ_P_STEP4
      }
#ifdef MPQ_TIMELINE
      if (todo == k1 - k0) MPQ_STAMP(7)
#endif
      if (++c == C || todo == 1) {
        // end of the tile (or of the wave's run): park the rows of the 2-bit part, added over the four
        // units of a block position in a fixed order, and batch column 0 of the 4-bit accumulator
        // (lane (j, 0) holds rows 4 j .. 4 j + 3)
        float yr = yacc;
        yr += __shfl_xor(yr, 16);
        yr += __shfl_xor(yr, 32);
        float* rt_ = red + t * (2 * W + 1) * 16;
        if (j == 0) rt_[wv * 16 + i] = yr;
        if (i == 0) *(float4_t*)(rt_ + (W + wv) * 16 + 4 * j) = acc4;
        yacc = 0.f;
        acc4 = float4_t{0.f, 0.f, 0.f, 0.f};
        c = 0;
        ++t;
      }
    }
  }
#undef MPQ_P_REQUEST
  MPQ_STAMP(8)
  MPQ_VMCNT(0);  // the re-requested blocks past the end of the run
  lds_barrier();
  MPQ_STAMP(9)

  // ---- (5) row r of tile t: 16 lanes add the 2 W partial sums and the outlier term, always in the same order
  for (uint32_t o = tid; o < 256u * n; o += W * 64u) {
    const uint32_t t = o >> 8, r = (o >> 4) & 15u, k = o & 15u;
    const float* rt0 = red + t * (2 * W + 1) * 16 + r;
    float sum = rt0[k * 16];
    if (W == 16) sum += rt0[(k + 16) * 16];
    if (k == 0) sum += rt0[2 * W * 16];
    sum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sum), 0x111, 0xf, 0xf, true));
    sum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sum), 0x112, 0xf, 0xf, true));
    sum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sum), 0x114, 0xf, 0xf, true));
    sum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sum), 0x118, 0xf, 0xf, true));
    const uint32_t row = (tile0 + t) * 16 + r;
    if (k == 15u && row < (uint32_t)b.N) a.Y[row] = half_to_bits((half_t)sum);
  }
  MPQ_STAMP(10)
  MPQ_TL_NOTE(11, k1 - k0)
  MPQ_TL_FLUSH(blockIdx.x, wv, W - 1, lane)
}

// ------------------------------------------------------------------------------------ dequant
//
// Row-major fp16 copy of the dense part: W_out[n][k] = fp16((code - z1) * s1), bit-exact eq. 5.
// A lane decodes its unit (64 or 32 columns of one row); the wave turns the decoded bytes through a small
// LDS area so that neighbouring lanes write contiguous bytes: eight lanes the 128 bytes of a (row, 2-bit
// unit), which are a whole line when a unit is one piece (first-order groups of 64 columns or more) and
// the unit's pieces otherwise; four lanes the 64 bytes of a (row, 4-bit unit).  Narrower groups go through
// mpq_dequant_lines_kernel below whenever their unit table fits its LDS; this kernel is what is left for them.
//
// The kernel writes 2 bytes per weight against 0.33 read; what was measured on the way to its shape:
//   - Loads and stores of a wave complete in one order, so a wait for a load that was requested after a
//     store also waits for that store, and a load that comes out of HBM while every compute unit streams
//     stores takes 5 to 25 microseconds.  Hence batches: a wave requests everything its next D blocks need
//     (table entries and code words, then the scale words the entries point at), and only then decodes
//     and stores those blocks with no load in between.  With the D blocks per wave that most matrices
//     leave, all reads of the launch happen before its first store.
//   - The store rounds read no memory: the table entry that says where a (row, unit) goes comes out of
//     the registers of the lane that decoded it (v_readlane; the unit is the same for the whole wave in a
//     round).  The stores are buffer stores on the tile's 16 output rows: rows past the end of the
//     matrix and padding pieces (offset 2 GiB) fail the range check and are dropped by the hardware,
//     so the rounds hold no branch.  Whole lines are written with the non-temporal bit when nothing reads
//     them back (NT: no outliers to add afterwards): 3 to 17 % faster; behind it the outlier pass is slower.
//   - No block depends on another: the blocks of the whole matrix (tile-major) are dealt round-robin over
//     all waves of a grid that is resident at once and a multiple of the number of compute units
//     (a compute unit with four workgroups where others have three ends a third later): wave w takes
//     blocks w, w + W, w + 2W, ... (dc, dt = W mod C, W div C: the step without a division).
//   - The outliers (dense + sparse, Sec. 2.3).  A second kernel that adds them to the finished matrix makes the
//     memory side read and write one 64-byte piece per outlier (22016 x 4096, 0.5 %: + 20 us).  ADD adds
//     them while the decoded block is in LDS: the tile's outlier block index names the words of (row, block),
//     lane (row r, j) takes words j and j + 4 of row r (both requested with the batch's other loads; further
//     ones, which are rare, with loads of their own), finds the piece by comparing the column with the first
//     columns of the block's pieces and adds in place (native fp16 add = the definition's fp32 add and one
//     rounding).
template <int PU, bool NT, bool AL = false, bool ADD = false>
__global__ void __launch_bounds__(256)
mpq_dequant_kernel(const DevBlob b, uint16_t* __restrict__ Wout, const int dc, const int dt, const int table_bytes) {
#pragma clang fp contract(off)
  MPQ_TL_DECL
  MPQ_STAMP(0)
  constexpr int PAIR = 144;  // LDS bytes per (row, unit): + 16 so that lanes fall into different banks
  constexpr int PU4 = PU > 1 ? PU / 2 : 1;
  constexpr int D = PU == 1 ? 8 : 4;      // blocks per batch (10 or 4 + 6 PU registers per block)
  __shared__ __align__(16) unsigned char turn[4][64 * PAIR];
  // the unit table, when it fits (K up to 28672 for one piece per unit): a wave's first requests then depend
  // on no other load, and go out before any wave of the launch has stored anything
  extern __shared__ __align__(16) unsigned char table[];  // table_bytes of it, or nothing
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, j = lane >> 4;
  const bool staged = table_bytes != 0;
  if (staged) {
    for (int o = tid * 16; o < 32 * PU * b.C; o += 256 * 16) *(uint4*)(table + o) = *(const uint4*)(b.units + o);
    __syncthreads();
  }
  const DecodeConsts kc = make_consts();
  unsigned char* mine = turn[wv];
  const uint32_t m1_lane = (uint32_t)i * 2u, m2_lane = b.off_m2 + ((uint32_t)i >> b.m2_shift) * 4u;
  uint4* dst = (uint4*)(mine + lane * PAIR);
  const int C = b.C, T = b.T;
  const uint32_t pad_entry = b.pad_entry;  // what bits 16-31 of a padding piece's table word hold
  const uint32_t row_bytes = 2u * (uint32_t)b.K;
  constexpr uint32_t DROPPED = 0x80000000u;  // beyond any tile's 16 rows (at most 2 MiB)
  // the wave's first block (tile, block of the tile) and how many it has
  const int waves = 4 * (int)gridDim.x, w0 = (int)blockIdx.x * 4 + wv;
  int t_pre = w0 / C, c_pre = w0 - t_pre * C;  // walks ahead of the blocks being decoded; stays on the wave's last block
  int left = t_pre < T ? (int)(((long long)T * C - w0 + waves - 1) / waves) : 0;
  uint4 qs[D];
  uint32_t m1s[D][PU], m2s[D][PU];
  uint2 es[D][PU];
  int ts[D], cs[D];
  uint32_t ofirst[D], ocount[D], oword[D][2];  // ADD: first word and number of words of (block, row i); words j and j + 4
  for (; left > 0; left -= D) {
#ifdef MPQ_TIMELINE
    // per wave, summed over its batches and blocks: [1] requests issued, [2] wait for a block's words, [3] decode,
    // turn and stores, [11] blocks
    const unsigned long long tl_r = __builtin_amdgcn_s_memrealtime();
#endif
    // ---- everything the next D blocks need (past the wave's last block: that block again, in bounds, not used)
#pragma unroll
    for (int d = 0; d < D; ++d) {
      ts[d] = t_pre;
      cs[d] = c_pre;
      const uint32_t ue = (uint32_t)(4 * c_pre + j) * (8 * PU);  // table entries of the lane's unit
#pragma unroll
      for (int q_ = 0; q_ < PU; ++q_) es[d][q_] = staged ? *(const uint2*)(table + ue + 8 * q_) : *(const uint2*)(b.units + ue + 8 * q_);
      qs[d] = ((const uint4*)(b.tiles + (size_t)t_pre * b.tile_stride + b.codes_off))[c_pre * 64 + lane];
      if constexpr (ADD) {
        // a 4-bit block: the entries of the last 2-bit block, and no words
        const int cx = c_pre < b.B2 ? c_pre : b.B2 - 1;
        const uint16_t* ox = (const uint16_t*)(b.tiles + (size_t)t_pre * b.tile_stride + b.off_oidx) + cx * 16 + i;
        ofirst[d] = ox[0];
        ocount[d] = ox[16];
      }
      int c2 = c_pre + dc, t2 = t_pre + dt;
      if (c2 >= C) { c2 -= C; ++t2; }
      if (t2 < T) { t_pre = t2; c_pre = c2; }
    }
    if constexpr (!AL) {
      // the words of its pieces' scales (first order: 8-bit quantized scale and zero point of the lane's row,
      // second order: scale and zero point of its row group)
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const unsigned char* side = b.tiles + (size_t)ts[d] * b.tile_stride;
#pragma unroll
        for (int q_ = 0; q_ < PU; ++q_) {
          m1s[d][q_] = *(const uint16_t*)(side + (m1_lane + (es[d][q_].y & 0xFFFFu)));
          m2s[d][q_] = *(const uint32_t*)(side + (m2_lane + (es[d][q_].y >> 16)));
        }
      }
    }
    if constexpr (ADD) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const uint32_t* words = (const uint32_t*)(b.tiles + (size_t)ts[d] * b.tile_stride + b.off_ot + MPQ_OTILE_HEAD);
        ocount[d] = cs[d] < b.B2 ? ocount[d] - ofirst[d] : 0u;
        const uint32_t w0 = ofirst[d] + (uint32_t)j, w1 = w0 + 4u;
        oword[d][0] = words[w0 < b.ocap ? w0 : 0u];
        oword[d][1] = words[w1 < b.ocap ? w1 : 0u];
      }
    }
#ifdef MPQ_TIMELINE
    tl_[1] += __builtin_amdgcn_s_memrealtime() - tl_r;
#endif
    // ---- decode, turn, store
#pragma unroll
    for (int d = 0; d < D; ++d) {
      if (d >= left) break;
      const int t_cur = ts[d], c_cur = cs[d];
      const bool two = c_cur < b.B2;
      const uint4 q = qs[d];
#ifdef MPQ_TIMELINE
      const unsigned long long tl_a = __builtin_amdgcn_s_memrealtime();
      if constexpr (!AL) asm volatile("" ::"v"(q.x), "v"(m1s[d][0]), "v"(m2s[d][0]));
      const unsigned long long tl_b = __builtin_amdgcn_s_memrealtime();
#endif
      const uint32_t lo[4] = {q.x, q.y, q.z, q.w};
      // the tile's 16 rows of the output as a buffer
      const int rows_left = b.N - t_cur * 16;
      const __amdgpu_buffer_rsrc_t out_rows = __builtin_amdgcn_make_buffer_rsrc(
          (unsigned char*)Wout + (size_t)t_cur * 16 * row_bytes, 0, (uint32_t)(rows_left < 16 ? rows_left : 16) * row_bytes, 0x00020000);
      // word W (x or y) of piece Q of unit U of the block: from the first lane that decoded that unit
#define MPQ_DQ_WORD(Q, W, U) (uint32_t)__builtin_amdgcn_readlane((int)es[d][Q].W, 16 * (U))
      // stores of one half: (row, unit) pairs 16*s .. 16*s + 15 in round s (= unit s), four lanes per pair
#define MPQ_DQ_STORE_HALF(HALF, SPP)                                                                      \
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); /* the wave's own LDS area: lanes run in lockstep */ \
  _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                                         \
    const int pair = (lane >> 2) + s * 16; /* lane index (unit * 16 + row) that decoded it */             \
    const int chunk = lane & 3, cg = (HALF) * 4 + chunk; /* step inside the half, inside the unit */      \
    constexpr int QA = ((HALF) * 4) / (SPP);             /* the piece of the half's first step */         \
    uint32_t ex = MPQ_DQ_WORD(QA, x, s), ey = MPQ_DQ_WORD(QA, y, s);                                      \
    if constexpr ((SPP) < 4) { /* two pieces per half */                                                  \
      constexpr int QB = QA + 1 < PU ? QA + 1 : QA;                                                       \
      const uint32_t exb = MPQ_DQ_WORD(QB, x, s), eyb = MPQ_DQ_WORD(QB, y, s);                            \
      if (chunk >> 1) { ex = exb; ey = eyb; }                                                             \
    }                                                                                                     \
    const uint4 v = *(const uint4*)(mine + pair * PAIR + chunk * 16);                                     \
    /* padding pieces point at the zero scale entries */                                                  \
    const uint32_t at = (ey >> 16) != pad_entry ? (uint32_t)(pair & 15) * row_bytes + ex + (uint32_t)(cg % (SPP)) * 16u : DROPPED; \
    __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{v.x, v.y, v.z, v.w}, out_rows, (int)at, 0, 0);         \
  }                                                                                                       \
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); /* reads done before the area is overwritten */
      // stores of a whole 2-bit unit: (row, unit) pairs 8*s .. 8*s + 7 in round s (unit s / 2), eight lanes per pair
#define MPQ_DQ_STORE_UNIT                                                                                 \
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                                      \
  _Pragma("unroll") for (int s = 0; s < 8; ++s) {                                                         \
    const int pair = (lane >> 3) + s * 8;                                                                 \
    const int ch = lane & 7; /* decode step = 16-byte chunk of the unit */                                \
    uint32_t ex = MPQ_DQ_WORD(0, x, s >> 1), ey = MPQ_DQ_WORD(0, y, s >> 1);                              \
    _Pragma("unroll") for (int q_ = 1; q_ < PU; ++q_) { /* the piece of the lane's step */                \
      const uint32_t exq = MPQ_DQ_WORD(q_, x, s >> 1), eyq = MPQ_DQ_WORD(q_, y, s >> 1);                  \
      if (ch / (8 / PU) == q_) { ex = exq; ey = eyq; }                                                    \
    }                                                                                                     \
    const uint4 v = *(const uint4*)(mine + pair * PAIR + ch * 16);                                        \
    const uint32_t at = (ey >> 16) != pad_entry ? (uint32_t)(pair & 15) * row_bytes + ex + (uint32_t)(ch % (8 / PU)) * 16u : DROPPED; \
    __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{v.x, v.y, v.z, v.w}, out_rows, (int)at, 0, NT ? 2 : 0); \
  }                                                                                                       \
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#define MPQ_DQ_PIECES(NP, FOUR)                                                               \
  half2_t s1p[NP];                                                                            \
  half_t zb[NP];                                                                              \
  if constexpr (AL) {                                                                         \
    uint2 ent_[NP];                                                                           \
    uint32_t xoff_[NP];                                                                       \
    _Pragma("unroll") for (int q_ = 0; q_ < NP; ++q_) ent_[q_] = es[d][q_];                   \
    pieces_aligned<NP, FOUR>(ent_, b.tiles + (size_t)t_cur * b.tile_stride, b, (uint32_t)i, s1p, zb, xoff_); \
  } else {                                                                                    \
    _Pragma("unroll") for (int q_ = 0; q_ < NP; ++q_) {                                       \
      const half_t s1_ = scale_dequant(m1s[d][q_] & 0xFFu, m2s[d][q_]); /* exactly 0 for a padding piece */ \
      s1p[q_] = half2_t{s1_, s1_};                                                            \
      zb[q_] = bits_to_half((uint16_t)(0x6400u | (m1s[d][q_] >> 8))); /* 1024 + z1 */         \
    }                                                                                         \
  }
#define MPQ_DQ_STEP8(P) dst[(P)] = decode_step<true, P>(lo, hi, s1p[(P) / (8 / PU)], zb[(P) / (8 / PU)], kc);
#define MPQ_DQ_STEP(TWO, P)                                                                   \
  {                                                                                           \
    constexpr int SPP = ((TWO) ? 8 : 4) / ((TWO) ? PU : PU4), Q = (P) / SPP;                  \
    dst[(P) & 3] = decode_step<TWO, P>(lo, hi, s1p[Q], zb[Q], kc);                            \
  }
      if (two) {
        MPQ_DQ_PIECES(PU, false)
        const uint32_t hi[4] = {rotr8(q.x), rotr8(q.y), rotr8(q.z), rotr8(q.w)};
        MPQ_DQ_STEP8(0) MPQ_DQ_STEP8(1) MPQ_DQ_STEP8(2) MPQ_DQ_STEP8(3)
        MPQ_DQ_STEP8(4) MPQ_DQ_STEP8(5) MPQ_DQ_STEP8(6) MPQ_DQ_STEP8(7)
        if constexpr (ADD) {
          // byte offsets of the first columns of the block's pieces in a row.  They are compared from the back, so
          // that the first match stays: padding pieces (offset 0) come after the real ones, and every word of
          // the block lies in a real one.
          constexpr uint32_t PB = 128u / PU;  // bytes of a piece in a row
          uint32_t px[4][PU];
#pragma unroll
          for (int u_ = 0; u_ < 4; ++u_) {
#pragma unroll
            for (int q_ = 0; q_ < PU; ++q_) px[u_][q_] = MPQ_DQ_WORD(q_, x, u_);
          }
          auto add_outlier = [&](const uint32_t word) {
            const uint32_t at = 2u * (word & 0xFFFFu);
            uint32_t where = 0xFFFFFFFFu;
#pragma unroll
            for (int u_ = 3; u_ >= 0; --u_) {
#pragma unroll
              for (int q_ = PU - 1; q_ >= 0; --q_) {
                const uint32_t dq = at - px[u_][q_];
                if (dq < PB) where = ((uint32_t)u_ * 16u + (uint32_t)i) * PAIR + (uint32_t)q_ * PB + dq;
              }
            }
            if (where != 0xFFFFFFFFu) {
              uint16_t* w16 = (uint16_t*)(mine + where);
              *w16 = half_to_bits(bits_to_half(*w16) + bits_to_half((uint16_t)(word >> 16)));
            }
          };
          if ((uint32_t)j < ocount[d]) add_outlier(oword[d][0]);
          if ((uint32_t)j + 4u < ocount[d]) add_outlier(oword[d][1]);
          if (ocount[d] > 8u) {  // more than eight outliers of a row in the block's columns
            const uint32_t* words = (const uint32_t*)(b.tiles + (size_t)t_cur * b.tile_stride + b.off_ot + MPQ_OTILE_HEAD);
            for (uint32_t e = 8u + (uint32_t)j; e < ocount[d]; e += 4u) add_outlier(words[ofirst[d] + e]);
          }
        }
        MPQ_DQ_STORE_UNIT
      } else {
        MPQ_DQ_PIECES(PU4, true)
        const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
        MPQ_DQ_STEP(false, 0) MPQ_DQ_STEP(false, 1) MPQ_DQ_STEP(false, 2) MPQ_DQ_STEP(false, 3)
        MPQ_DQ_STORE_HALF(0, 4 / PU4)
      }
#undef MPQ_DQ_STEP
#undef MPQ_DQ_STEP8
#undef MPQ_DQ_PIECES
#undef MPQ_DQ_STORE_UNIT
#undef MPQ_DQ_STORE_HALF
#undef MPQ_DQ_WORD
#ifdef MPQ_TIMELINE
      tl_[2] += tl_b - tl_a;
      tl_[3] += __builtin_amdgcn_s_memrealtime() - tl_b;
      tl_[11] += 1;
#endif
    }
  }
  MPQ_STAMP(4)
  MPQ_TL_NOTE(12, __builtin_amdgcn_s_getreg((31 << 11) | 4))   // HW_ID: where the wave ran
  MPQ_TL_NOTE(13, __builtin_amdgcn_s_getreg((31 << 11) | 20))  // XCC_ID
  MPQ_TL_FLUSH(blockIdx.x, wv, 3, lane)
}

// Dequantization where a group is narrower than a 128-byte line of the output (groups of 16 or 32 columns).
// There a line holds pieces of several units, 2-bit and 4-bit ones, that lie far apart in the code streams.
// Written piece by piece the memory side sees 32- and 64-byte fragments whose other parts come from other waves
// at other times: a 32-byte half of a 64-byte segment that finds its other half gone from the L2 costs a
// read-modify-write (measured: 1.9 TB/s instead of 4.5 to 5.4), and such fragments cannot carry the non-temporal
// bit, which is worth a third.  So a workgroup here owns 16 rows x KC columns of the output: its waves decode
// every unit that has a piece in those columns (both streams are in K order: the pieces of a column range are a
// range of each stream, found by bisection of the unit table once per workgroup) into an LDS image of the
// output, add the outliers there (the address is the column, no search), and write whole lines, 1 KiB of a row per
// instruction, non-temporal.  Units that straddle a range are decoded by both neighbours, each keeping its own
// pieces.  The requests of a range go out while the range before the previous one is stored (two register sets).
template <int PU, bool AL, bool ADD, int KC, int TB>
__global__ void __launch_bounds__(256)
mpq_dequant_lines_kernel(const DevBlob b, uint16_t* __restrict__ Wout, const int np2, const int np4, const uint32_t pad_y2,
                         const uint32_t pad_y4) {
#pragma clang fp contract(off)
  constexpr int PP2 = PU, PP4 = PU > 1 ? PU / 2 : 1;  // pieces of a 2-bit and of a 4-bit unit
  constexpr int ROWB = 2 * KC + 16;                   // bytes of a row of the image: + 16 so that rows start in different banks
  constexpr int D = 4;                                // passes of a wave whose words are requested together
  constexpr uint32_t DROPPED = 0x80000000u;
  __shared__ __align__(16) unsigned char out[16 * ROWB];
  __shared__ __align__(16) unsigned char table[TB];
  __shared__ uint16_t cut2[68], cut4[68];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, j = lane >> 4;
  for (int o = tid * 16; o < 32 * PU * b.C; o += 256 * 16) *(uint4*)(table + o) = *(const uint4*)(b.units + o);
  __syncthreads();
  // cut[k] = the first piece of the stream whose first column is not before column k KC
  const int nch = (b.K + KC - 1) / KC;
  for (int idx = tid; idx < 2 * (nch + 1); idx += 256) {
    const int four = idx > nch, k = four ? idx - nch - 1 : idx;
    const uint32_t x_k = (uint32_t)k * (2u * KC);
    int lo = 0, hi = four ? np4 : np2;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      const uint32_t at = four ? (uint32_t)(4 * b.B2 + mid / PP4) * (8 * PU) + 8u * (uint32_t)(mid % PP4)
                               : (uint32_t)(mid / PP2) * (8 * PU) + 8u * (uint32_t)(mid % PP2);
      if (*(const uint32_t*)(table + at) < x_k) lo = mid + 1;
      else hi = mid;
    }
    (four ? cut4 : cut2)[k] = (uint16_t)lo;
  }
  __syncthreads();
  const DecodeConsts kc = make_consts();
  const uint32_t m1_lane = (uint32_t)i * 2u, m2_lane = b.off_m2 + ((uint32_t)i >> b.m2_shift) * 4u;
  const uint32_t row_bytes = 2u * (uint32_t)b.K;
  const int total = b.T * nch;
  const int orow = tid >> 4, om = tid & 15;  // outliers: 16 threads per row, the rows of a wave are the ones it stores

  // What a wave holds of one range between its requests and its decode: two such sets, so that the requests of the
  // range after the next are on their way while this one is decoded and stored (a load that leaves while every
  // compute unit streams stores takes 5 to 25 microseconds; the four matrices of a Llama2-7B layer with their
  // input from memory: 139 -> 119 us with byte-wide, 157 -> 146 us with aligned metadata).
  struct Set {
    uint4 qs[D];
    uint32_t at[D][PU];  // where the piece starts in the lane's row of the image (aligned metadata: | position in its triple); DROPPED: no piece
    uint32_t ma[D][PU], mb[D][PU], mc[D][AL ? PU : 1];
    bool live[D], two[D];
    uint32_t ofirst, ocount, oword[2];
  };

  // requests what passes wv + 4 (d + D * batch), d = 0 .. D - 1, of the range need
  auto request = [&](Set& r, const int item, const int batch) {
    const int t = item / nch, k = item - t * nch;
    const int c2lo = __builtin_amdgcn_readfirstlane(cut2[k]), c2hi = __builtin_amdgcn_readfirstlane(cut2[k + 1]);
    const int c4lo = __builtin_amdgcn_readfirstlane(cut4[k]), c4hi = __builtin_amdgcn_readfirstlane(cut4[k + 1]);
    const int u2lo = c2lo / PP2, n2u = c2hi > c2lo ? (c2hi + PP2 - 1) / PP2 - u2lo : 0, p2 = (n2u + 3) >> 2;
    const int u4lo = c4lo / PP4, n4u = c4hi > c4lo ? (c4hi + PP4 - 1) / PP4 - u4lo : 0, p4 = (n4u + 3) >> 2;
    const unsigned char* side = b.tiles + (size_t)t * b.tile_stride;
    const uint32_t x0 = (uint32_t)k * (2u * KC);
    uint32_t ys[D][PU];
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const int pass = wv + 4 * (d + D * batch);
      r.live[d] = pass < p2 + p4;
      r.two[d] = pass < p2;
      if (!r.live[d]) continue;
      const int ulo = r.two[d] ? u2lo : u4lo, nu = r.two[d] ? n2u : n4u, pp = r.two[d] ? PP2 : PP4;
      const int clo = r.two[d] ? c2lo : c4lo, chi = r.two[d] ? c2hi : c4hi;
      const int v = ulo + 4 * (r.two[d] ? pass : pass - p2) + j, vv = v < ulo + nu ? v : ulo;  // a unit past the range's: its first, no piece kept
      const int vb = r.two[d] ? vv : 4 * b.B2 + vv;  // place in the table and in the tile's code blocks
      const uint32_t ue = (uint32_t)vb * (8 * PU);
#pragma unroll
      for (int q_ = 0; q_ < PU; ++q_) {
        const int idx = v * pp + q_;
        const uint2 e = *(const uint2*)(table + ue + 8 * (q_ < pp ? q_ : 0));
        const bool mine = q_ < pp && idx >= clo && idx < chi;
        ys[d][q_] = mine ? e.y : (r.two[d] ? pad_y2 : pad_y4);
        r.at[d][q_] = mine ? ((uint32_t)i * ROWB + (e.x - x0)) | (AL ? e.y & 3u : 0u) : DROPPED;
      }
      r.qs[d] = ((const uint4*)(side + b.codes_off))[(vb >> 2) * 64 + (vb & 3) * 16 + i];
    }
    if constexpr (ADD) {
      if (batch == 0) {
        const int cA = c2lo / (4 * PP2), cB = c2hi > c2lo ? (c2hi - 1) / (4 * PP2) + 1 : cA;
        const uint16_t* ox = (const uint16_t*)(side + b.off_oidx) + orow;
        r.ofirst = ox[cA * 16];
        r.ocount = ox[cB * 16];
      }
    }
#pragma unroll
    for (int d = 0; d < D; ++d) {
      if (!r.live[d]) continue;
#pragma unroll
      for (int q_ = 0; q_ < PU; ++q_) {
        const uint32_t y = ys[d][q_];
        if constexpr (AL) {
          const uint32_t idx = (y >> 16) + ((uint32_t)i >> b.m2_shift);
          r.ma[d][q_] = r.two[d] ? (uint32_t)*(const uint16_t*)(side + (y & 0xFFFCu) + 2u * (uint32_t)i)
                                 : (uint32_t)*(const uint8_t*)(side + b.off_m1b + (y & 0xFFFFu) + (uint32_t)i);
          r.mb[d][q_] = *(const uint16_t*)(side + b.off_s2 + 2u * idx);
          r.mc[d][q_] = *(const uint8_t*)(side + b.off_z2 + idx);
        } else {
          r.ma[d][q_] = *(const uint16_t*)(side + (m1_lane + (y & 0xFFFFu)));
          r.mb[d][q_] = *(const uint32_t*)(side + (m2_lane + (y >> 16)));
        }
      }
    }
    if constexpr (ADD) {
      if (batch == 0) {
        const uint32_t* words = (const uint32_t*)(side + b.off_ot + MPQ_OTILE_HEAD);
        r.ocount -= r.ofirst;
        const uint32_t w0 = r.ofirst + (uint32_t)om, w1 = w0 + 16u;
        r.oword[0] = words[w0 < b.ocap ? w0 : 0u];
        r.oword[1] = words[w1 < b.ocap ? w1 : 0u];
      }
    }
  };

  // decodes the requested passes into the image
  auto decode = [&](const Set& r) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      if (!r.live[d]) continue;
      const uint4 q = r.qs[d];
      const uint32_t lo[4] = {q.x, q.y, q.z, q.w};
      half2_t s1p[PU];
      half_t zb[PU];
      uint32_t at[PU];
#pragma unroll
      for (int q_ = 0; q_ < PU; ++q_) {
        uint32_t s_int, z1, m2 = 0;
        at[q_] = r.at[d][q_];
        if constexpr (AL) {
          const uint32_t w = r.ma[d][q_];
          if (r.two[d]) {
            const uint32_t pos = at[q_] & 3u;
            z1 = (w >> (2u * pos)) & 3u;
            s_int = pos == 0 ? (w >> 6) & 15u : (w >> (pos == 1 ? 10u : 13u)) & 7u;
          } else {
            s_int = w & 15u;
            z1 = w >> 4;
          }
          if (at[q_] != DROPPED) at[q_] &= ~3u;
        } else {
          s_int = r.ma[d][q_] & 0xFFu;
          z1 = r.ma[d][q_] >> 8;
          m2 = r.mb[d][q_];
        }
        const half_t s1 = AL ? scale_dequant_int_zero(s_int, r.mc[d][AL ? q_ : 0], r.mb[d][q_]) : scale_dequant(s_int, m2);
        s1p[q_] = half2_t{s1, s1};
        zb[q_] = bits_to_half((uint16_t)(0x6400u | z1));  // 1024 + z1
      }
#define MPQ_DL_STEP(TWO, P)                                                                      \
  {                                                                                              \
    constexpr int SPP = (TWO) ? 8 / PP2 : 4 / PP4, Q = (P) / SPP;                                \
    const uint4 v = decode_step<TWO, P>(lo, hi, s1p[Q], zb[Q], kc);                              \
    if (at[Q] != DROPPED) *(uint4*)(out + at[Q] + ((P) % SPP) * 16) = v;                         \
  }
      if (r.two[d]) {
        const uint32_t hi[4] = {rotr8(q.x), rotr8(q.y), rotr8(q.z), rotr8(q.w)};
        MPQ_DL_STEP(true, 0) MPQ_DL_STEP(true, 1) MPQ_DL_STEP(true, 2) MPQ_DL_STEP(true, 3)
        MPQ_DL_STEP(true, 4) MPQ_DL_STEP(true, 5) MPQ_DL_STEP(true, 6) MPQ_DL_STEP(true, 7)
      } else {
        const uint32_t hi[4] = {q.x >> 8, q.y >> 8, q.z >> 8, q.w >> 8};
        MPQ_DL_STEP(false, 0) MPQ_DL_STEP(false, 1) MPQ_DL_STEP(false, 2) MPQ_DL_STEP(false, 3)
      }
#undef MPQ_DL_STEP
    }
  };

  // one range: decode, the set's next requests, outliers, stores
  const int step = (int)gridDim.x;
  auto range = [&](Set& r, const int item) {
    const int t = item / nch, k = item - t * nch;
    decode(r);
    {  // ranges of more than 16 passes (most of a long range 4-bit)
      const int c2lo = cut2[k], c2hi = cut2[k + 1], c4lo = cut4[k], c4hi = cut4[k + 1];
      const int n2u = c2hi > c2lo ? (c2hi + PP2 - 1) / PP2 - c2lo / PP2 : 0, n4u = c4hi > c4lo ? (c4hi + PP4 - 1) / PP4 - c4lo / PP4 : 0;
      const int passes = ((n2u + 3) >> 2) + ((n4u + 3) >> 2);
      for (int batch = 1; batch * 4 * D < passes; ++batch) {  // (leaves the set's outlier words alone)
        request(r, item, batch);
        decode(r);
      }
    }
    lds_barrier();
    const uint32_t x0 = (uint32_t)k * (2u * KC);
    const uint32_t of_cur = r.ofirst, oc_cur = r.ocount, ow0 = r.oword[0], ow1 = r.oword[1];
    if (item + 2 * step < total) request(r, item + 2 * step, 0);
    if constexpr (ADD) {
      auto add_outlier = [&](const uint32_t word) {
        const uint32_t rel = (word & 0xFFFFu) - (uint32_t)k * KC;
        if (rel < (uint32_t)KC) {
          uint16_t* w16 = (uint16_t*)(out + orow * ROWB + 2u * rel);
          *w16 = half_to_bits(bits_to_half(*w16) + bits_to_half((uint16_t)(word >> 16)));
        }
      };
      if ((uint32_t)om < oc_cur) add_outlier(ow0);
      if ((uint32_t)om + 16u < oc_cur) add_outlier(ow1);
      if (oc_cur > 32u) {
        const uint32_t* words = (const uint32_t*)(b.tiles + (size_t)t * b.tile_stride + b.off_ot + MPQ_OTILE_HEAD);
        for (uint32_t e = 32u + (uint32_t)om; e < oc_cur; e += 16u) add_outlier(words[of_cur + e]);
      }
    }
    // the wave's four rows, 1 KiB per instruction
    const int rows_left = b.N - t * 16;
    const __amdgpu_buffer_rsrc_t out_rows = __builtin_amdgcn_make_buffer_rsrc(
        (unsigned char*)Wout + (size_t)t * 16 * row_bytes, 0, (uint32_t)(rows_left < 16 ? rows_left : 16) * row_bytes, 0x00020000);
    const uint32_t cb = row_bytes - x0 < 2u * KC ? row_bytes - x0 : 2u * KC;  // bytes of a row in this range
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const uint32_t row = (uint32_t)(4 * wv + rr);
#pragma unroll
      for (int n = 0; n < 2 * KC / 1024; ++n) {
        const uint32_t o = (uint32_t)n * 1024u + (uint32_t)lane * 16u;
        const uint4 v = *(const uint4*)(out + row * ROWB + o);
        const uint32_t at = o < cb ? row * row_bytes + x0 + o : DROPPED;
        __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{v.x, v.y, v.z, v.w}, out_rows, (int)at, 0, 2);
      }
    }
    lds_barrier();
  };

  Set sa, sb;
  int item = blockIdx.x;
  if (item < total) request(sa, item, 0);
  if (item + step < total) request(sb, item + step, 0);
  for (; item < total; item += 2 * step) {
    range(sa, item);
    if (item + step < total) range(sb, item + step);
  }
}

// W[row][col] = fp16(W[row][col] + val) for every outlier word of the tile (native fp16 add = the
// fp32 add followed by one rounding that the definition states); 16 threads per row.
static __global__ void __launch_bounds__(256)
mpq_outlier_add_kernel(const DevBlob b, uint16_t* __restrict__ Wout) {
  const int orow = threadIdx.x >> 4, oq = threadIdx.x & 15;
  const int row = blockIdx.x * 16 + orow;
  if (row >= b.N) return;
  const uint32_t* rec = (const uint32_t*)(b.tiles + (size_t)blockIdx.x * b.tile_stride + b.off_ot);
  const uint32_t* words = rec + MPQ_OTILE_HEAD / 4;
  const int32_t rp0 = (int32_t)rec[orow], rp1 = (int32_t)rec[orow + 1];
  for (int32_t e = rp0 + oq; e < rp1; e += 16) {
    const uint32_t word = words[e];
    uint16_t* at = Wout + (size_t)row * b.K + (word & 0xFFFFu);
    const half_t s = bits_to_half(*at) + bits_to_half((uint16_t)(word >> 16));
    *at = half_to_bits(s);
  }
}

// ------------------------------------------------------------------------------------ bandwidth reference
//
// Reads `n16` 16-byte words once and does nothing else: what the memory system delivers to a kernel of
// this size and launch pattern, the figure the product kernels' throughput is set against.  Every
// workgroup walks its own contiguous part, eight 16-byte loads per lane in flight.
static __global__ void __launch_bounds__(256)
mpq_stream_kernel(const uint4* __restrict__ src, const size_t n16, uint32_t* __restrict__ sink) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x, hi = lo + per < n16 ? lo + per : n16;
  uint32_t acc = 0;
  size_t i = lo + threadIdx.x;
  for (; i + 1792 < hi; i += 2048) {  // eight loads per lane in flight
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + 256 * u];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < hi; i += 256) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9E3779B9u && sink) *sink = acc;  // keeps the loads alive; practically never taken
}

// ------------------------------------------------------------------------------------ host side

namespace {

const mpq_plan kAutoPlan = {};

// Launch status of THIS launch only, from the launch call's own return value: the library neither reads nor
// clears the thread's last-error state, so an error some earlier HIP call of the caller left behind is not
// reported as ours and is still there for the caller to find.
template <typename T>
struct SameType {
  using type = T;
};
template <typename... KArgs>
inline hipError_t launch_kernel(void (*kernel)(KArgs...), const dim3 grid, const dim3 block, const size_t lds_bytes, hipStream_t stream,
                                typename SameType<KArgs>::type... args) {
  void* ptrs[] = {(void*)&args...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, stream);
}
#define MPQ_LAUNCH(...)                                                   \
  do {                                                                    \
    if (launch_kernel(__VA_ARGS__) != hipSuccess) return MPQ_ERR_HIP;     \
  } while (0)

mpq_status make_dev(const void* hdr_host, const void* blob_dev, MpqHeader* h, DevBlob* d) {
  if (!hdr_host || !blob_dev) return MPQ_ERR_NULL;
  mpq_status st = mpq_internal_check_header(hdr_host, h);
  if (st != MPQ_OK) return st;
  if (((uintptr_t)blob_dev & 15u) != 0) return MPQ_ERR_ALIGN;
  const unsigned char* p = (const unsigned char*)blob_dev;
  d->tiles = p + h->off_tiles;
  d->units = p + h->off_units;
  d->tile_stride = (uint32_t)h->tile_stride;
  d->side_bytes = (uint32_t)h->side_bytes;
  d->codes_off = (uint32_t)h->codes_off;
  d->off_m2 = 32u * ((uint32_t)h->G + 1);
  d->off_ot = d->off_m2 + (uint32_t)mpq_meta2_bytes(h);
  d->off_m1b = d->off_s2 = d->off_z2 = 0;
  d->pad_entry = mpq_meta2_zero(h);
  if (h->meta == MPQ_META_PAPER) {
    d->off_m1b = mpq_p_off_m1b(h);
    d->off_s2 = mpq_p_off_s2(h);
    d->off_z2 = mpq_p_off_z2(h);
    d->off_ot = mpq_p_off_outl(h);
    d->pad_entry = mpq_p_zero_entry(h);
  }
  d->m2_shift = 0;  // g2_axis 0: one pair per row; g2_axis 1: one pair per block of g2 rows
  if (h->g2_axis == 1)
    for (int g = h->g2 < MPQ_TILE_ROWS ? h->g2 : MPQ_TILE_ROWS; g > 1; g >>= 1) ++d->m2_shift;
  d->off_oidx = (uint32_t)h->oidx_off;
  d->ocap = (uint32_t)h->ocap;
  d->N = h->N; d->K = h->K; d->G = h->G; d->S = h->S; d->B2 = h->B2; d->C = h->B2 + h->B4; d->T = h->T;
  if (h->tile_stride > 0xFFFFFFFFull) return MPQ_ERR_UNSUPPORTED;
  return MPQ_OK;
}

// Compute units of the current device; the work splits are sized by it.
mpq_status cu_count(int* cus) {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      n <= 0)
    return MPQ_ERR_HIP;
  *cus = n;
  return MPQ_OK;
}

struct Ctx {  // what every launcher needs
  const MpqHeader& h;
  const DevBlob& d;
  const mpq_plan& plan;
  mpq_report* report;
  int cus;
  hipStream_t s;
};

void note(const Ctx& c, int kernel, int launches, int waves, int tiles, long workgroups) {
  if (!c.report) return;
  c.report->kernel = kernel;
  c.report->launches += launches;
  c.report->waves = waves;
  c.report->tiles_per_workgroup = tiles;
  c.report->workgroups = (int32_t)workgroups;
}

// LDS bytes the batch kernel needs for M rows at ring depth PD: ring, reduction slots, two
// side-record buffers, unit table, activation rows.
size_t mm_lds_bytes(const MpqHeader& h, int M, int PD, int waves = 4) {
  const size_t NT = M > 16 ? 2 : 1;
  return (size_t)waves * PD * 1024 + waves * NT * 1024 + 2 * h.side_bytes + 32ull * mpq_pu2(h.g1) * (h.B2 + h.B4) +
         (size_t)M * (2ull * h.K + 16);
}

constexpr size_t kLdsPerCu = 160 * 1024;  // LDS of one gfx950 compute unit
// Static LDS size of which three workgroups fit a compute unit: 52 KiB (of 53 KiB only two do: measured, the
// third workgroup of 10240 x 8192 waited for a place and the launch took 7 % longer).
#define MPQ_LDS_THIRD (52 * 1024)

// ---------------------------------------------------------------- M = 1, per-weight decode kernel

// LDS bytes of the GEMV kernel: ring, partial sums, n side records, unit table, activations.
size_t gemv_lds_bytes(const MpqHeader& h, int PD, int waves, int n) {
  return (size_t)waves * PD * 1024 + (size_t)n * (waves + 1) * 64 + (size_t)n * h.side_bytes +
         32ull * mpq_pu2(h.g1) * (h.B2 + h.B4) + 2ull * h.K;
}

// n = the most tiles a workgroup gets; the kernel deals the tiles evenly to the grid's workgroups.
template <int PD, int LDSB, int WV, int PU, bool AL = false>
mpq_status launch_gemv(const Ctx& c, const uint16_t* X, uint16_t* Y, int n, unsigned grid) {
  const uint32_t n_lo = (uint32_t)c.h.T / grid, n_more = (uint32_t)c.h.T - n_lo * grid;
  if (n_lo + (n_more ? 1u : 0u) > (uint32_t)n) return MPQ_ERR_UNSUPPORTED;
  MPQ_LAUNCH((mpq_gemv_kernel<PD, LDSB, WV, PU, AL>), dim3(grid), dim3(WV * 64), 0, c.s, c.d.tiles, c.d.units, X, c.d.tile_stride,
             c.d.side_bytes, c.d.codes_off, (uint32_t)c.d.C, (uint32_t)c.d.K, (uint32_t)n, n_lo, n_more, c.d, Y);
  note(c, MPQ_KERNEL_GEMV_DECODE, 1, WV, n, grid);
  return MPQ_OK;
}

// GEMV with WV waves per workgroup and n tiles per workgroup in the smallest LDS class that holds
// it.  Two code blocks per wave in flight: deeper rings were measured and change nothing.
template <int WV, int PU, bool AL = false>
mpq_status gemv_class(const Ctx& c, const uint16_t* X, uint16_t* Y, int n, unsigned grid) {
  const size_t need = gemv_lds_bytes(c.h, 2, WV, n);
  if (need <= 32 * 1024) return launch_gemv<2, 32 * 1024, WV, PU, AL>(c, X, Y, n, grid);
  if (need <= 40 * 1024) return launch_gemv<2, 40 * 1024, WV, PU, AL>(c, X, Y, n, grid);
  if (need <= MPQ_LDS_THIRD) return launch_gemv<2, MPQ_LDS_THIRD, WV, PU, AL>(c, X, Y, n, grid);
  if (need <= 80 * 1024) return launch_gemv<2, 80 * 1024, WV, PU, AL>(c, X, Y, n, grid);
  if (need <= 160 * 1024) return launch_gemv<2, 160 * 1024, WV, PU, AL>(c, X, Y, n, grid);
  return MPQ_ERR_UNSUPPORTED;
}

template <int WV>
mpq_status gemv_waves(const Ctx& c, const uint16_t* X, uint16_t* Y, int n, unsigned grid) {
  switch (mpq_pu2(c.h.g1)) {  // first-order groups per 2-bit unit
    case 1: return gemv_class<WV, 1>(c, X, Y, n, grid);
    case 2: return gemv_class<WV, 2>(c, X, Y, n, grid);
    default: return c.h.meta == MPQ_META_PAPER ? gemv_class<WV, 4, true>(c, X, Y, n, grid) : gemv_class<WV, 4>(c, X, Y, n, grid);
  }
}

// Work split of the per-weight GEMV (waves per workgroup, tiles per workgroup), from measurements on
// the Llama2-7B / Llama3-8B / Llama2-70B shapes:
//   - up to 1.5 tiles per compute unit: 16 waves on one tile, so that every SIMD has several waves;
//   - else 8 waves on one tile if four such workgroups fit a compute unit (all 32 wave slots busy
//     and the most workgroups to balance);
//   - else (long rows: the staged activations crowd the LDS) 16 waves on two tiles when the
//     workgroups still spread evenly over the compute units, which halves the staging per tile.
mpq_status gemv_decode(const Ctx& c, const uint16_t* X, uint16_t* Y) {
  const MpqHeader& h = c.h;
  int waves, n = 1;
  if (2 * h.T <= 3 * c.cus) {
    waves = 16;
  } else if (gemv_lds_bytes(h, 2, 8, 1) <= 40 * 1024) {
    waves = 8;
  } else {
    const int half = (h.T + 1) / 2;
    if ((half % c.cus == 0 || half >= 4 * c.cus) && gemv_lds_bytes(h, 2, 16, 2) <= kLdsPerCu) {
      waves = 16;
      n = 2;
    } else {
      waves = gemv_lds_bytes(h, 2, 8, 1) <= MPQ_LDS_THIRD ? 8 : 16;
    }
  }
  if (c.plan.gemv_waves > 0) waves = c.plan.gemv_waves;
  if (c.plan.gemv_tiles > 0) n = c.plan.gemv_tiles > 8 ? 8 : c.plan.gemv_tiles;
  while (n > 1 && gemv_lds_bytes(h, 2, waves, n) > kLdsPerCu) --n;
  const unsigned grid = (unsigned)((h.T + n - 1) / n);
  if (waves == 16) {
    const mpq_status st = gemv_waves<16>(c, X, Y, n, grid);
    if (st != MPQ_ERR_UNSUPPORTED) return st;
  }
  return gemv_waves<8>(c, X, Y, n, grid);
}

// ---------------------------------------------------------------- M = 1, plane-sum kernel

// LDS layout of the plane-sum GEMV for n tiles per workgroup of W waves; false if it does not fit.
bool plane_layout(const MpqHeader& h, uint32_t W, uint32_t PD, uint32_t n, bool x_lds, uint32_t budget, PlanePlan* pl) {
  const uint32_t C = (uint32_t)(h.B2 + h.B4);
  uint32_t off = W * PD * 1536u;                        // ring: PD slots of codes + two meta words per lane
  pl->off_park = off;   off += n * (2u * W + 1u) * 64u;
  pl->off_units = off;  off += 32u * C;                  // unit table
  off = (off + 15u) & ~15u;
  pl->off_xs = off;     off += x_lds ? (2u * (uint32_t)h.K + 15u) & ~15u : 256u * (uint32_t)h.B4;
  pl->x_lds = x_lds ? 1u : 0u;
  pl->off_utab = off;   off += 32u * (uint32_t)h.B2;     // 8 bytes per 2-bit unit
  pl->off_pieces = off; off += 768u * (uint32_t)h.B2;    // 192 bytes per 2-bit unit
  pl->off_zero = off;   off += 128u;
  pl->obuf_bytes = MPQ_OTILE_HEAD + 4u * (uint32_t)h.ocap;
  pl->off_obuf = off;   off += n * pl->obuf_bytes;
  pl->n = n;
  return off <= budget;
}

// Share of a SIMD's blocks per age rank of its waves, in sixteenths (see PlanePlan): `older` = what the
// oldest wave of a SIMD takes beyond an even share, handed down linearly to the youngest.
void plane_deal(uint32_t W, int older, PlanePlan* pl) {
  const uint32_t ranks = W / 4u;
  uint32_t share[4] = {0, 0, 0, 0};
  if (ranks == 4) {
    const uint32_t d = older < 0 ? 0u : older > 3 ? 3u : (uint32_t)older;   // 4+d, 4+d/2.., 4-d/2.., 4-d
    share[0] = 4u + d; share[1] = 4u + d / 2u; share[2] = 4u - d / 2u; share[3] = 4u - d;
  } else {
    const uint32_t d = older < 0 ? 0u : older > 6 ? 6u : (uint32_t)older;
    share[0] = 8u + d; share[1] = 8u - d;
  }
  pl->cum[0] = 0;
  for (uint32_t w = 0; w < 16; ++w) pl->cum[w + 1] = pl->cum[w] + (w < W ? share[w / 4u] : 0u);
}

template <int LDSB, int WV>
mpq_status launch_planes(const Ctx& c, PlaneArgs& a) {
  const unsigned grid = (unsigned)((c.h.T + a.pl.n - 1) / a.pl.n);
  MPQ_LAUNCH((mpq_gemvp_kernel<LDSB, WV>), dim3(grid), dim3(WV * 64), 0, c.s, a);
  note(c, MPQ_KERNEL_GEMV_PLANES, 1, WV, (int)a.pl.n, grid);
  return MPQ_OK;
}

// The plane-sum kernel needs one first-order group per unit (g1 >= 64) and room in the LDS for the
// split activations; MPQ_ERR_UNSUPPORTED otherwise.
mpq_status gemv_planes(const Ctx& c, const uint16_t* X, uint16_t* Y) {
  const MpqHeader& h = c.h;
  PlaneArgs a;
  if (mpq_pu2(h.g1) != 1 || 4 * (h.B2 + h.B4) > MPQ_PLANE_MAX_UNITS || !mpq_internal_unit_words(&h, a.uw))
    return MPQ_ERR_UNSUPPORTED;
  const uint32_t W = c.plan.gemv_waves == 8 ? 8u : 16u;
  // tiles per workgroup: one generation of workgroups if the LDS allows it, at most W (a wave group per
  // tile sums its outliers), else the smallest number of equal generations
  uint32_t n = 0;
  if (c.plan.gemv_tiles > 0) {
    n = (uint32_t)c.plan.gemv_tiles > W ? W : (uint32_t)c.plan.gemv_tiles;
    if (!plane_layout(h, W, 2, n, true, 160 * 1024, &a.pl) && !plane_layout(h, W, 2, n, false, 160 * 1024, &a.pl)) return MPQ_ERR_UNSUPPORTED;
  } else {
    // the whole activation vector on chip if it fits next to its fp8 pieces, else (K = 28672) only the pieces
    for (uint32_t gens = 1;; ++gens) {
      n = ((uint32_t)h.T + gens * (uint32_t)c.cus - 1u) / (gens * (uint32_t)c.cus);
      if (n <= W && (plane_layout(h, W, 2, n, true, 160 * 1024, &a.pl) || plane_layout(h, W, 2, n, false, 160 * 1024, &a.pl))) break;
      if (n <= 1) return MPQ_ERR_UNSUPPORTED;
    }
  }
  plane_deal(W, c.plan.gemv_older > 0 ? c.plan.gemv_older - 1 : 2, &a.pl);
  a.b = c.d;
  a.X = X;
  a.Y = Y;
  const uint32_t need = a.pl.off_obuf + a.pl.n * a.pl.obuf_bytes;
  if (W == 16) return need <= 80 * 1024 ? launch_planes<80 * 1024, 16>(c, a) : launch_planes<160 * 1024, 16>(c, a);
  return need <= 80 * 1024 ? launch_planes<80 * 1024, 8>(c, a) : launch_planes<160 * 1024, 8>(c, a);
}

// ---------------------------------------------------------------- 2 <= M <= 32

// Persistent batch kernel with WV waves per workgroup; one or two workgroups per compute unit.
template <int NT, int PD, int LDSB, int WV, int PU = 1, bool AL = false>
mpq_status launch_batch(const Ctx& c, const uint16_t* X, uint16_t* Y, int M) {
  size_t per_cu = kLdsPerCu / LDSB;
  if (per_cu * WV > 32) per_cu = 32 / WV;
  if (per_cu < 1) per_cu = 1;
  long grid = (long)c.cus * (long)per_cu;
  if (c.plan.max_workgroups > 0 && grid > c.plan.max_workgroups) grid = c.plan.max_workgroups;
  if (grid > c.h.T) grid = c.h.T;
  MPQ_LAUNCH((mpq_mm_kernel<NT, PD, LDSB, WV, PU, AL>), dim3((unsigned)grid), dim3(WV * 64), 0, c.s, c.d, X, Y, M);
  note(c, MPQ_KERNEL_BATCH_RESIDENT, 1, WV, 0, grid);
  return MPQ_OK;
}

// Persistent batch kernel with 4 waves per workgroup (the most workgroups per compute unit).
template <int NT, int PD, int LDSB, int PU = 1, bool AL = false>
mpq_status launch_mm(const Ctx& c, const uint16_t* X, uint16_t* Y, int M) {
  size_t per_cu = kLdsPerCu / LDSB;  // as many workgroups as fit at once (LDS, 32 waves per compute unit)
  if (per_cu > 8) per_cu = 8;
  if (per_cu < 1) per_cu = 1;
  long grid = (long)c.cus * (long)per_cu;
  if (c.plan.max_workgroups > 0 && grid > c.plan.max_workgroups) grid = c.plan.max_workgroups;
  if (grid > c.h.T) grid = c.h.T;
  MPQ_LAUNCH((mpq_mm_kernel<NT, PD, LDSB, 4, PU, AL>), dim3((unsigned)grid), dim3(256), 0, c.s, c.d, X, Y, M);
  note(c, MPQ_KERNEL_BATCH_RESIDENT, 1, 4, 0, grid);
  return MPQ_OK;
}

// Static LDS size classes of the product kernel; each has the ring depth that keeps enough bytes
// in flight for the number of workgroups that fit a compute unit.
template <int NT>
mpq_status mm_chunk(const Ctx& c, const uint16_t* X, uint16_t* Y, int M) {
  const MpqHeader& h = c.h;
  const int bw = c.plan.batch_waves;
  if (mpq_pu2(h.g1) > 1) {
    // first-order groups shorter than a unit (g1 = 16, 32): persistent workgroups in a few classes
    const bool four = mpq_pu2(h.g1) == 4, al = h.meta == MPQ_META_PAPER;  // the aligned metadata comes with g1 = 16
#define MPQ_PIECES(CALL2, CALL4, CALL4A) return !four ? CALL2 : al ? CALL4A : CALL4
    if (mm_lds_bytes(h, M, 2, 8) <= 80 * 1024)
      MPQ_PIECES((launch_batch<NT, 2, 80 * 1024, 8, 2>(c, X, Y, M)), (launch_batch<NT, 2, 80 * 1024, 8, 4>(c, X, Y, M)),
                 (launch_batch<NT, 2, 80 * 1024, 8, 4, true>(c, X, Y, M)));
    if (mm_lds_bytes(h, M, 3, 8) <= 160 * 1024)
      MPQ_PIECES((launch_batch<NT, 3, 160 * 1024, 8, 2>(c, X, Y, M)), (launch_batch<NT, 3, 160 * 1024, 8, 4>(c, X, Y, M)),
                 (launch_batch<NT, 3, 160 * 1024, 8, 4, true>(c, X, Y, M)));
    if (mm_lds_bytes(h, M, 3) <= 160 * 1024)
      MPQ_PIECES((launch_mm<NT, 3, 160 * 1024, 2>(c, X, Y, M)), (launch_mm<NT, 3, 160 * 1024, 4>(c, X, Y, M)),
                 (launch_mm<NT, 3, 160 * 1024, 4, true>(c, X, Y, M)));
#undef MPQ_PIECES
    return MPQ_ERR_UNSUPPORTED;
  }
  if (bw != 4) {
    // many waves share one copy of the activations: 16 (or 8) waves per workgroup
    if (bw != 8) {
      if (mm_lds_bytes(h, M, 2, 16) <= 80 * 1024) return launch_batch<NT, 2, 80 * 1024, 16>(c, X, Y, M);
      // one workgroup of 16 waves per compute unit, unless two of 8 waves fit and the matrix has the
      // tiles to feed them: two independent workgroups lose less at the barriers of every tile
      // (measured: 13-14 % on the 12288x4096 and 22016x4096 matrices at M = 4)
      const bool two_of_8 = bw == 0 && mm_lds_bytes(h, M, 2, 8) <= 80 * 1024 && 2 * h.T >= 3 * c.cus;
      if (!two_of_8 && mm_lds_bytes(h, M, 2, 16) <= 160 * 1024) return launch_batch<NT, 2, 160 * 1024, 16>(c, X, Y, M);
    }
    if (mm_lds_bytes(h, M, 2, 8) <= MPQ_LDS_THIRD) return launch_batch<NT, 2, MPQ_LDS_THIRD, 8>(c, X, Y, M);
    if (mm_lds_bytes(h, M, 2, 8) <= 80 * 1024) return launch_batch<NT, 2, 80 * 1024, 8>(c, X, Y, M);
    if (mm_lds_bytes(h, M, 3, 8) <= 160 * 1024) return launch_batch<NT, 3, 160 * 1024, 8>(c, X, Y, M);
  }
  if (mm_lds_bytes(h, M, 3) <= 32 * 1024) return launch_mm<NT, 3, 32 * 1024>(c, X, Y, M);
  if (mm_lds_bytes(h, M, 3) <= 40 * 1024) return launch_mm<NT, 3, 40 * 1024>(c, X, Y, M);
  if (mm_lds_bytes(h, M, 4) <= MPQ_LDS_THIRD) return launch_mm<NT, 4, MPQ_LDS_THIRD>(c, X, Y, M);
  if (mm_lds_bytes(h, M, 6) <= 80 * 1024) return launch_mm<NT, 6, 80 * 1024>(c, X, Y, M);
  if (mm_lds_bytes(h, M, 8) <= 160 * 1024) return launch_mm<NT, 8, 160 * 1024>(c, X, Y, M);
  if (mm_lds_bytes(h, M, 3) <= 160 * 1024) return launch_mm<NT, 3, 160 * 1024>(c, X, Y, M);
  return MPQ_ERR_UNSUPPORTED;
}

// Plan of the large-batch kernel: staged rows XR, the fewest ranges H whose activations fit the LDS of a
// workgroup of W waves next to ring, unit table and park area, NB tile bands so that H * NB
// workgroups about fill the compute units, groups of at most R = 8 tiles.
bool plan_slices(const MpqHeader& h, const mpq_plan& plan, int cus_i, int M, uint32_t W, uint32_t budget, SlicePlan* pl,
                 int* XR_out) {
  const uint32_t PU = (uint32_t)mpq_pu2(h.g1);
  const uint32_t MW = h.meta == MPQ_META_PAPER ? 3u : 2u;  // dwords of scale words per lane and piece in a ring slot
  const uint32_t NT = M > 16 ? 2 : 1, XR = M <= 8 ? 8 : 16 * NT;
  const uint32_t B2 = (uint32_t)h.B2, B4 = (uint32_t)h.B4;
  const uint32_t maxH = B2 > B4 ? B2 : B4;
  const uint32_t cus = (uint32_t)cus_i;
  uint32_t off = W * 2u * (1024u + 256u * MW * PU);
  pl->off_units = off; off += (32u * PU * (B2 + B4) + 15u) & ~15u;
  pl->off_park = off;  off += W * 2048u;
  off = (off + 1023u) & ~1023u;
  pl->off_xbuf = off;
  if (off >= budget) return false;
  uint32_t H = plan.lb_min_ranges > 1 ? (uint32_t)plan.lb_min_ranges : 1u;
  if (H > maxH) H = maxH;
  for (; H <= maxH && H <= cus; ++H) {
    const uint32_t nb2 = (B2 + H - 1) / H, nb4 = (B4 + H - 1) / H;  // the largest range
    if ((size_t)(nb2 * 512u + nb4 * 256u) * XR > budget - off) continue;
    uint32_t NB = cus / H;
    if (NB > (uint32_t)h.T) NB = (uint32_t)h.T;
    pl->H = (int32_t)H;
    pl->older16 = plan.lb_older16 > 0 && plan.lb_older16 < 16 ? (uint32_t)plan.lb_older16 : 10u;
    pl->NB = (int32_t)NB;
    pl->R = plan.lb_tiles > 0 && plan.lb_tiles <= 8 ? plan.lb_tiles : 8;
    *XR_out = (int)XR;
    return true;
  }
  return false;
}

// Workspace of the large-batch kernel: partial sums P[H][T][16 NT][16] fp32, then the transposed
// activations XT[K][XR] fp16.
size_t slice_workspace_bytes(const MpqHeader& h, const SlicePlan& pl, int NT, int XR, size_t* p_bytes) {
  *p_bytes = ((size_t)pl.H * (size_t)h.T * NT * 256 * sizeof(float) + 255) & ~(size_t)255;
  return *p_bytes + (size_t)h.K * XR * sizeof(uint16_t);
}

mpq_status launch_slices(const Ctx& c, const uint16_t* X, uint16_t* Y, int M, void* ws, size_t ws_bytes) {
  const MpqHeader& h = c.h;
  const DevBlob& d = c.d;
  hipStream_t s = c.s;
  SlicePlan pl;
  int XR = 0;
  const int NT = M > 16 ? 2 : 1;
  // 8 waves per workgroup leave the most LDS for the activations and 256 registers per lane (the B
  // operands of a position and up to 8 x NT accumulators stay in registers); 16 waves, with half
  // the registers and a third less LDS for the activations, measured equal or slower on every shape
  const int pu = mpq_pu2(h.g1);
  if (!plan_slices(h, c.plan, c.cus, M, 8, 160 * 1024, &pl, &XR)) return MPQ_ERR_UNSUPPORTED;
  size_t p_bytes = 0;
  if (!ws || ((uintptr_t)ws & 255u) != 0 || ws_bytes < slice_workspace_bytes(h, pl, NT, XR, &p_bytes)) return MPQ_ERR_UNSUPPORTED;
  unsigned char* scratch = (unsigned char*)ws;
  float* P = (float*)scratch;
  uint16_t* XT = (uint16_t*)(scratch + p_bytes);
  const dim3 grid((unsigned)(pl.H * pl.NB));
#define MPQ_LAUNCH_S(NTV, XRV, WV, PUV) \
  MPQ_LAUNCH((mpq_mms_kernel<NTV, XRV, 160 * 1024, WV, PUV>), grid, dim3(WV * 64), 0, s, d, X, P, XT, M, pl)
#define MPQ_LAUNCH_S8(PUV) \
  { if (XR == 8) MPQ_LAUNCH_S(1, 8, 8, PUV); else if (NT == 1) MPQ_LAUNCH_S(1, 16, 8, PUV); else MPQ_LAUNCH_S(2, 32, 8, PUV); }
  if (pu == 1) MPQ_LAUNCH_S8(1) else if (pu == 2) MPQ_LAUNCH_S8(2) else if (h.meta != MPQ_META_PAPER) MPQ_LAUNCH_S8(4)
  else {
#define MPQ_LAUNCH_SA(NTV, XRV) \
  MPQ_LAUNCH((mpq_mms_kernel<NTV, XRV, 160 * 1024, 8, 4, true>), grid, dim3(8 * 64), 0, s, d, X, P, XT, M, pl)
    if (XR == 8) MPQ_LAUNCH_SA(1, 8); else if (NT == 1) MPQ_LAUNCH_SA(1, 16); else MPQ_LAUNCH_SA(2, 32);
#undef MPQ_LAUNCH_SA
  }
#undef MPQ_LAUNCH_S8
#undef MPQ_LAUNCH_S
  // from here on Y is undefined if the second launch fails: the first kernel is already enqueued
  const dim3 fgrid((unsigned)h.T), fblock(256);
  if (XR == 8) MPQ_LAUNCH((mpq_mms_finish_kernel<1, 8>), fgrid, fblock, 0, s, d, XT, P, Y, M, pl.H, (uint32_t)h.ocap);
  else if (NT == 1) MPQ_LAUNCH((mpq_mms_finish_kernel<1, 16>), fgrid, fblock, 0, s, d, XT, P, Y, M, pl.H, (uint32_t)h.ocap);
  else MPQ_LAUNCH((mpq_mms_finish_kernel<2, 32>), fgrid, fblock, 0, s, d, XT, P, Y, M, pl.H, (uint32_t)h.ocap);
  note(c, MPQ_KERNEL_BATCH_RANGES, 2, 8, pl.R, (long)pl.H * pl.NB);
  return MPQ_OK;
}

// Which batch-1 kernel: the plane-sum kernel pays a fixed price per workgroup (the activations are split
// into fp8 pieces, two more barriers) and needs 40 % fewer vector instructions per block; measured on
// the Llama2-7B / Llama3-8B / Llama2-70B shapes it wins from about 200 code blocks per compute unit on
// (57344 x 8192, 504 blocks: 35 against 41 us; 128256 x 4096, 595: 42 against 46 us) and loses below
// (12288 x 4096, 54 blocks: 8.7 against 7.0 us; 28672 x 4096, 133: 13.0 against 12.1 us).  Rows too
// long to stage the activations next to their pieces (8192 x 28672: 24.2 against 23.2 us, the split then
// reads them from memory) stay with the per-weight kernel unless a plan asks otherwise.
mpq_status gemv_all(const Ctx& c, const uint16_t* X, uint16_t* Y) {
  const bool planes = c.plan.gemv_path == 1 || (c.plan.gemv_path == 0 && c.h.K <= 16384 &&
                                                (int64_t)c.h.T * (c.h.B2 + c.h.B4) >= 200ll * c.cus);
  if (planes) {
    const mpq_status st = gemv_planes(c, X, Y);
    if (st != MPQ_ERR_UNSUPPORTED || c.plan.gemv_path == 1) return st;
  }
  return gemv_decode(c, X, Y);
}

mpq_status mm_all(const Ctx& c, const uint16_t* X, uint16_t* Y, int M, void* ws, size_t ws_bytes) {
  const MpqHeader& h = c.h;
  if (M == 1) return gemv_all(c, X, Y);
  if (mm_lds_bytes(h, 1, 3) > kLdsPerCu) return MPQ_ERR_UNSUPPORTED;
  int Mc = M;  // largest batch chunk whose activations fit LDS together with everything else
  while (Mc > 1 && mm_lds_bytes(h, Mc, 3) > kLdsPerCu) --Mc;
  if (Mc > 16 && Mc < M) Mc = 16;
  {
    // The large-batch kernel reads and decodes the weights once whatever M is and costs about 1.25 x
    // the matrix-vector product plus 4-12 us for its second kernel; the chunked path below costs one
    // pass over the weights per chunk and a per-column outlier loop that weighs from M = 9 on.
    // Measured on the Llama2-7B and Llama2-70B shapes, M = 2..32, outlier fractions 0 / 0.5 / 1.5 %:
    // up to M = 8 the large-batch kernel wins from three chunks on, and with two chunks unless the
    // matrix is small; above, whenever there are two chunks or the matrix is not small.  "Small" is below 12 MB,
    // and below 24 MB where the whole batch fits next to 8 or 16 waves in one chunk (M = 9 to 14 at K = 4096:
    // 12288 x 4096, 17.7 MB, 13.4-13.9 us with 16 waves and 15.3 with 8 against 16.3-16.5 us; 22016 x 4096, 31.7 MB,
    // 23.1-23.8 and 26.2 against 23.8-24.4 us).
    const int chunks = (M + Mc - 1) / Mc;
    // (groups of 16 or 32 columns: 8 waves; 12288 x 4096 at M = 12 with groups of 16, 22.8 MB: 16.6 against 18.7 us)
    const bool many_waves = (mpq_pu2(h.g1) == 1 && mm_lds_bytes(h, M, 2, 16) <= 160 * 1024) || mm_lds_bytes(h, M, 3, 8) <= 160 * 1024;
    // With the aligned metadata the K-range kernel gathers three words per piece instead of two and the bounds are
    // 24 and 40 MB (22016 x 4096, 33.5 MB, at M = 12: 28.3 against 31.6 us; 12288 x 4096, 18.7 MB, at M = 16: 20.4
    // against 21.7; 4096 x 11008, 16.7 MB, at M = 8 in two chunks: 20.3 against 22.5).
    const bool al = h.meta == MPQ_META_PAPER;
    const bool large = h.total_bytes >= ((M > 8 && chunks == 1 && many_waves ? (al ? 40u : 24u) : (al ? 24u : 12u)) << 20);
    // one chunk that leaves room for four waves only (M = 8 at K = 8192): 10240 x 8192, 25 MB, 24.9 against 20.5 us;
    // 8192 x 8192, 20 MB, 18.1 against 17.9; 4096 x 11008 at M = 5, 15.5 MB, 12.8 against 15.3
    const bool four_waves = mpq_pu2(h.g1) == 1 && chunks == 1 && !many_waves && h.total_bytes >= (20u << 20);
    const bool better = M <= 8 ? chunks >= 3 || (chunks == 2 && large) || four_waves : chunks >= 2 || large;
    if (c.plan.large_batch == 0 ? better : c.plan.large_batch > 0) {
      const mpq_status st = launch_slices(c, X, Y, M, ws, ws_bytes);
      if (st != MPQ_ERR_UNSUPPORTED) return st;
    }
  }
  {
    const int chunks = (M + Mc - 1) / Mc;
    Mc = (M + chunks - 1) / chunks;  // chunks of about equal size (8 rows as 4 + 4, not 7 + 1)
  }
  for (int m0 = 0; m0 < M; m0 += Mc) {
    const int mc = M - m0 < Mc ? M - m0 : Mc;
    const uint16_t* Xc = X + (size_t)m0 * h.K;
    uint16_t* Yc = Y + (size_t)m0 * h.N;
    mpq_status st = mc > 16 ? mm_chunk<2>(c, Xc, Yc, mc) : mm_chunk<1>(c, Xc, Yc, mc);
    if (st != MPQ_OK) return st;
  }
  return MPQ_OK;
}

}  // namespace

extern "C" {

mpq_status mpq_gemm_planned(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev, uint16_t* Y_dev,
                            int32_t M, void* workspace_dev, size_t workspace_bytes, void* stream, const mpq_plan* plan,
                            mpq_report* report) {
  if (report) memset(report, 0, sizeof(*report));
  if (!X_dev || !Y_dev) return MPQ_ERR_NULL;
  if (M < 1 || M > MPQ_MAX_M) return MPQ_ERR_SHAPE;
  MpqHeader h;
  DevBlob d;
  mpq_status st = make_dev(hdr_host, blob_dev, &h, &d);
  if (st != MPQ_OK) return st;
  if ((((uintptr_t)X_dev | (uintptr_t)Y_dev) & 15u) != 0) return MPQ_ERR_ALIGN;
  int cus = 0;
  if ((st = cu_count(&cus)) != MPQ_OK) return st;
  const Ctx c{h, d, plan ? *plan : kAutoPlan, report, cus, (hipStream_t)stream};
  return mm_all(c, X_dev, Y_dev, M, workspace_dev, workspace_bytes);
}

mpq_status mpq_gemm(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev, uint16_t* Y_dev,
                    int32_t M, void* workspace_dev, size_t workspace_bytes, void* stream) {
  return mpq_gemm_planned(hdr_host, blob_dev, X_dev, Y_dev, M, workspace_dev, workspace_bytes, stream, nullptr, nullptr);
}

// ---- mpq_gemm for callers that cannot hand over a workspace: the partial sums and the transposed
// activations of the K-range kernel go to an array that is part of the library's device image.
// In host code the array's name is only a stand-in: its device address is asked for once per device
// (with that device current) and kept; only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[MPQ_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_addr[kMaxDevices];  // device address of `scratch` on each device, once known

static mpq_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MPQ_ERR_HIP;
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MPQ_ERR_HIP;
    g_scratch_addr[dev].store(p, std::memory_order_release);  // every thread that asks gets the same answer
  }
  *out = p;
  return MPQ_OK;
}
}  // namespace

mpq_status mpq_gemm_static(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev, uint16_t* Y_dev,
                           int32_t M, void* stream) {
  size_t need = 0;
  mpq_status st = mpq_gemm_workspace_size_planned(hdr_host, M, nullptr, &need);
  if (st != MPQ_OK) return st;
  if (need > (size_t)MPQ_STATIC_SCRATCH_BYTES) return MPQ_ERR_SIZE;
  void* ws = nullptr;
  if (need > 0 && (st = static_scratch(&ws)) != MPQ_OK) return st;
  // nothing in the array has to start at zero: the kernels write every partial sum before it is read
  return mpq_gemm_planned(hdr_host, blob_dev, X_dev, Y_dev, M, ws, need > 0 ? (size_t)MPQ_STATIC_SCRATCH_BYTES : 0, stream,
                          nullptr, nullptr);
}

mpq_status mpq_gemm_workspace_size_planned(const void* hdr_host, int32_t M, const mpq_plan* plan, size_t* bytes) {
  if (!hdr_host || !bytes) return MPQ_ERR_NULL;
  if (M < 1 || M > MPQ_MAX_M) return MPQ_ERR_SHAPE;
  MpqHeader h;
  mpq_status st = mpq_internal_check_header(hdr_host, &h);
  if (st != MPQ_OK) return st;
  int cus = 0;
  if ((st = cu_count(&cus)) != MPQ_OK) return st;
  *bytes = 0;
  SlicePlan pl;
  int XR = 0;
  size_t p_bytes = 0;
  if (M > 1 && plan_slices(h, plan ? *plan : kAutoPlan, cus, M, 8, 160 * 1024, &pl, &XR))
    *bytes = slice_workspace_bytes(h, pl, M > 16 ? 2 : 1, XR, &p_bytes);
  return MPQ_OK;
}

mpq_status mpq_gemm_workspace_size(const void* hdr_host, int32_t M, size_t* bytes) {
  return mpq_gemm_workspace_size_planned(hdr_host, M, nullptr, bytes);
}

mpq_status mpq_gemv(const void* hdr_host, const void* blob_dev, const uint16_t* x_dev, uint16_t* y_dev,
                    void* stream) {
  return mpq_gemm_planned(hdr_host, blob_dev, x_dev, y_dev, 1, nullptr, 0, stream, nullptr, nullptr);
}

mpq_status mpq_gemv_multi(int32_t count, const void* const* hdr_host, const void* const* blob_dev,
                          const uint16_t* const* x_dev, uint16_t* const* y_dev, void* stream) {
  if (!hdr_host || !blob_dev || !x_dev || !y_dev) return MPQ_ERR_NULL;
  if (count < 1 || count > MPQ_MAX_MULTI) return MPQ_ERR_SHAPE;
  MultiArgs a;
  memset(&a, 0, sizeof(a));
  a.count = count;
  size_t need = 0;
  int pu = 0;
  uint64_t meta = 0;
  for (int p = 0; p < count; ++p) {
    if (!x_dev[p] || !y_dev[p]) return MPQ_ERR_NULL;
    MpqHeader h;
    mpq_status st = make_dev(hdr_host[p], blob_dev[p], &h, &a.b[p]);
    if (st != MPQ_OK) return st;
    if ((((uintptr_t)x_dev[p] | (uintptr_t)y_dev[p]) & 15u) != 0) return MPQ_ERR_ALIGN;
    if (p > 0 && (mpq_pu2(h.g1) != pu || h.meta != meta)) return MPQ_ERR_UNSUPPORTED;  // one kernel for all of them
    pu = mpq_pu2(h.g1);
    meta = h.meta;
    const size_t lds = gemv_lds_bytes(h, 2, 8, 1);
    need = lds > need ? lds : need;
    a.X[p] = x_dev[p];
    a.Y[p] = y_dev[p];
    a.first[p + 1] = a.first[p] + (uint32_t)h.T;
  }
  const dim3 grid(a.first[count]), block(8 * 64);
  hipStream_t s = (hipStream_t)stream;
#define MPQ_MULTI_CLASS(BYTES)                                                                          \
  if (need <= (BYTES)) {                                                                                \
    if (pu == 1) MPQ_LAUNCH((mpq_gemv_multi_kernel<2, (BYTES), 8, 1>), grid, block, 0, s, a);           \
    else if (pu == 2) MPQ_LAUNCH((mpq_gemv_multi_kernel<2, (BYTES), 8, 2>), grid, block, 0, s, a);      \
    else if (meta != MPQ_META_PAPER) MPQ_LAUNCH((mpq_gemv_multi_kernel<2, (BYTES), 8, 4>), grid, block, 0, s, a); \
    else MPQ_LAUNCH((mpq_gemv_multi_kernel<2, (BYTES), 8, 4, true>), grid, block, 0, s, a);             \
    return MPQ_OK;                                                                                      \
  }
  MPQ_MULTI_CLASS(40 * 1024)
  MPQ_MULTI_CLASS(80 * 1024)
  MPQ_MULTI_CLASS(160 * 1024)
#undef MPQ_MULTI_CLASS
  return MPQ_ERR_UNSUPPORTED;
}

#ifdef MPQ_TIMELINE
// Timeline build only: where the batch-1 kernels write their phase stamps (NULL = nowhere).  buf_dev: device
// memory of 2 x 16 x 8 bytes per workgroup of the launches that follow.  Synchronous.
mpq_status mpq_timeline_buffer(void* buf_dev) {
  return hipMemcpyToSymbol(HIP_SYMBOL(mpq_timeline_buf), &buf_dev, sizeof(buf_dev)) == hipSuccess ? MPQ_OK : MPQ_ERR_HIP;
}
#endif

mpq_status mpq_stream_probe(const void* src_dev, size_t bytes, uint32_t* sink_dev, void* stream) {
  if (!src_dev) return MPQ_ERR_NULL;
  if (((uintptr_t)src_dev & 15u) != 0) return MPQ_ERR_ALIGN;
  if (bytes < 16) return MPQ_ERR_SIZE;
  int cus = 0;
  mpq_status st = cu_count(&cus);
  if (st != MPQ_OK) return st;
  const size_t n16 = bytes / 16;
  size_t grid = (n16 + 1023) / 1024;            // at least 16 KiB per workgroup
  if (grid > (size_t)cus * 8) grid = (size_t)cus * 8;
  MPQ_LAUNCH(mpq_stream_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, (const uint4*)src_dev, n16, sink_dev);
  return MPQ_OK;
}

mpq_status mpq_dequant(const void* hdr_host, const void* blob_dev, uint16_t* W_out_dev, int add_outliers,
                       void* stream) {
  if (!W_out_dev) return MPQ_ERR_NULL;
  MpqHeader h;
  DevBlob d;
  mpq_status st = make_dev(hdr_host, blob_dev, &h, &d);
  if (st != MPQ_OK) return st;
  if (((uintptr_t)W_out_dev & 15u) != 0) return MPQ_ERR_ALIGN;
  int cus = 0;
  if ((st = cu_count(&cus)) != MPQ_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  const int pu = mpq_pu2(h.g1);
  // every block of the matrix dealt over the waves of at most four workgroups per compute unit (what 37 KiB
  // of LDS leave resident), the same number on every compute unit, as few as leave a wave at most one batch
  const long long blocks = (long long)h.T * (h.B2 + h.B4);
  if (blocks == 0) return MPQ_OK;
  const int batch = pu == 1 ? 8 : 4;
  // the unit table in LDS when it leaves three workgroups on a compute unit (four when it is at most 4 KiB)
  const int table_all = 32 * pu * (h.B2 + h.B4);
  const int table_bytes = table_all <= 16384 ? table_all : 0;
  const int fit = table_bytes <= 4096 ? 4 : 3;
  long long per_cu = (blocks + 4ll * batch * cus - 1) / (4ll * batch * cus);
  per_cu = per_cu > fit ? fit : per_cu;
  const dim3 grid((unsigned)(per_cu * cus));
  const int items = h.B2 + h.B4;
  const int dc = (int)((4ll * grid.x) % items), dt = (int)((4ll * grid.x) / items);
  const bool add = add_outliers && h.nnz > 0;
  const bool in_lds = add && h.oidx_off != 0;  // the blob has the outlier block index
  // Groups narrower than a line of the output: workgroups that own 16 rows x 2048 columns and write whole lines,
  // two of them on a compute unit (64 KiB of output image and up to 14 KiB of unit table each).
  constexpr int KC = 2048, TB = 14336;
  const int nch = (h.K + KC - 1) / KC;
  if (pu >= 2 && table_all <= TB && nch <= 64) {
    const int np2 = (int)h.n2, np4 = (int)h.n4;  // pieces of the two streams = groups
    // word 1 of the table entry of a piece that is not there (the packer's padding pieces hold the same)
    const uint32_t py2 = h.meta == MPQ_META_PAPER ? (32u * mpq_p_triples(&h)) | (mpq_p_zero_entry(&h) << 16)
                                                  : (32u * (uint32_t)h.G) | (mpq_meta2_zero(&h) << 16);
    const uint32_t py4 = h.meta == MPQ_META_PAPER ? (16u * (uint32_t)h.n4) | (mpq_p_zero_entry(&h) << 16) : py2;
    const long long total = (long long)h.T * nch;
    const dim3 lgrid((unsigned)(total < 2ll * cus ? total : 2ll * cus));
#define MPQ_DL_LAUNCH(PUV, ALV, ADDV) \
  MPQ_LAUNCH((mpq_dequant_lines_kernel<PUV, ALV, ADDV, KC, TB>), lgrid, dim3(256), 0, s, d, W_out_dev, np2, np4, py2, py4)
    if (pu == 2) { if (in_lds) MPQ_DL_LAUNCH(2, false, true); else MPQ_DL_LAUNCH(2, false, false); }
    else if (h.meta == MPQ_META_PAPER) { if (in_lds) MPQ_DL_LAUNCH(4, true, true); else MPQ_DL_LAUNCH(4, true, false); }
    else { if (in_lds) MPQ_DL_LAUNCH(4, false, true); else MPQ_DL_LAUNCH(4, false, false); }
#undef MPQ_DL_LAUNCH
    if (add && !in_lds) MPQ_LAUNCH(mpq_outlier_add_kernel, dim3(h.T), dim3(256), 0, s, d, W_out_dev);
    return MPQ_OK;
  }
  // One piece per unit, and rows too long for the above.  Lines are whole and carry the non-temporal bit where
  // nothing reads them back; with four pieces per unit they are fragments, which it would slow down.
#define MPQ_DQ_LAUNCH(...) \
  MPQ_LAUNCH((mpq_dequant_kernel<__VA_ARGS__>), grid, dim3(256), (size_t)table_bytes, s, d, W_out_dev, dc, dt, table_bytes)
  if (in_lds && pu == 1) MPQ_DQ_LAUNCH(1, true, false, true);
  else if (in_lds && pu == 2) MPQ_DQ_LAUNCH(2, true, false, true);
  else if (in_lds && h.meta == MPQ_META_PAPER) MPQ_DQ_LAUNCH(4, false, true, true);
  else if (in_lds) MPQ_DQ_LAUNCH(4, false, false, true);
  else if (pu == 1) { if (add) MPQ_DQ_LAUNCH(1, false); else MPQ_DQ_LAUNCH(1, true); }
  else if (pu == 2) { if (add) MPQ_DQ_LAUNCH(2, false); else MPQ_DQ_LAUNCH(2, true); }
  else if (h.meta == MPQ_META_PAPER) MPQ_DQ_LAUNCH(4, false, true);
  else MPQ_DQ_LAUNCH(4, false);
#undef MPQ_DQ_LAUNCH
  // Outliers of tiles without a block index (dense + sparse, Sec. 2.3): a second kernel.  Adding them at the end
  // of the first one, by the workgroup that wrote the weights, needs workgroups that own tiles and wait for their
  // stores, which costs more than the second launch (22016 x 4096, 0.5 % outliers: 82 us against 63 us).
  if (add && !in_lds) MPQ_LAUNCH(mpq_outlier_add_kernel, dim3(h.T), dim3(256), 0, s, d, W_out_dev);
  return MPQ_OK;
}

}  // extern "C"
