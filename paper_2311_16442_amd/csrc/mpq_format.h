// mpq_format.h - private description of the packed blob (shared by the host packer and the kernels).
//
// The blob follows the paper's memory-alignment rule (Sec. 3.3 "Memory Alignment"): the codes are
// split into two matrices, one per bit width, so that what one thread loads is one aligned vector
// unit holding codes of a single width.  The unit here is the widest per-lane load of gfx950,
// 16 bytes: 64 two-bit codes or 32 four-bit codes, always of one row and of consecutive columns.
//
// Rows are tiled by 16 (MPQ_TILE_ROWS) and units by 4 along K, so that one 64-lane wavefront load
// of 1 KiB ("block") is contiguous and covers 16 rows x 4 units with lane = unit_in_block*16 + row
// - the operand order of the 16x16x32 MFMA, which the small-batch product uses directly and the
// matrix-vector product reads equally well.
//
// A unit always holds codes of one bit width, but for first-order groups shorter than a unit
// (g1 = 16 or 32) it holds several groups: a "piece" is the part of a unit that belongs to one
// group - PU2 = max(1, 64/g1) pieces per 2-bit unit, PU4 = max(1, 32/g1) per 4-bit unit.  The
// pieces of a unit are consecutive groups of the unit's STREAM (all 2-bit groups in K order, or all
// 4-bit groups in K order), so they need not be neighbours in K; every piece covers whole decode
// steps of 8 columns.  For g1 >= 64 a unit is one piece (a half or quarter of a group).
//
//   header    256 B                       (MpqHeader; its last 112 bytes are the bitmap of the 4-bit K-groups)
//   units     2 x uint32 [4*(B2+B4)][PU2] per unit in stream order (2-bit units, then 4-bit units)
//                                         and per piece, ready for the kernels (a 4-bit unit uses
//                                         the first PU4 of its PU2 slots):
//                 word 0 = byte offset of the piece's first activation in an fp16 row (2*k0)
//                 word 1 = meta1 offset | meta2 offset << 16: byte offsets of the group's entry
//                          inside the tile's meta1 / meta2 arrays (before the per-lane part)
//                 a padding piece (stream padded to whole blocks, unused slots) has word 0 = 0
//                 and points at the extra all-zero last entries of meta1 / meta2: its scale
//                 decodes to exactly 0 without any test in the kernel
//   tiles     T x tile_stride B           one self-contained record per 16-row tile, so that a
//                                         workgroup finds everything it needs at one base address:
//       side (side_bytes):
//         meta1   (G+1) x 16 x 2 B  (s_int | z1 << 8) per (stream group, row); stream group order = all
//                                 2-bit groups in K order, then all 4-bit groups, then one zero entry
//         meta2   (s2 | z2 << 16), 4 B each, then one zero entry; mpq_meta2_bytes() in all:
//                   g2_axis 0: (S+1) x 16, per (super-group along K, row); lane part = 4*row
//                   g2_axis 1: (G+1) x nsub, per (stream group, block of g2 rows inside the tile),
//                              nsub = max(1, 16/g2) (g2 divides 16 or is a multiple of 16);
//                              lane part = 4*(row / g2) (0 for g2 >= 16)
//         outl    128 + 4*ocap B  uint32 start[17] (then zeros up to 128 B): start[r] = index of the first
//                                 word of row r of the tile, start[16] = number of words; then
//                                 uint32 word[ocap] = col | val << 16 (Sec. 2.3: one 32-bit word per
//                                 outlier, one 32-bit running count per row), rows in order;
//                                 ocap = the largest number of outliers in any tile, rounded up to 32.
//                                 A kernel can request a tile's outliers without first reading a
//                                 row pointer: no dependent load.
//       codes at codes_off (128-byte aligned): (B2 + B4) x 64 x 16 B, the 2-bit blocks then the 4-bit
//                                 blocks of the tile, [block][lane] 16-byte units
//       oidx at oidx_off (64-byte aligned; only for 0 < ocap <= 65535):
//                                 uint16 [B2 + 1][16]: entry [c][r] = index, among the tile's outlier words, of
//                                 the first word of row r whose column lies in 2-bit block c or a later one
//                                 ([B2][r] = end of row r).  The 2-bit stream is in K order and outliers live
//                                 in 2-bit groups only (Sec. 4.3), so the words of (row r, block c) are
//                                 [c][r] .. [c + 1][r] - 1: whoever decodes a block finds its outliers with two
//                                 loads and no search.  Derived from the outlier record; not counted as stored bits.
//
// Bit positions inside a unit (4 little-endian dwords).  A decode step P covers the 8 columns
// k0 + 8P .. k0 + 8P + 7; column 8P + 2d + h (d = 0..3, h = 0, 1) lives in dword d, in its low (h = 0)
// or high (h = 1) half-word, so that one mask applied to a dword isolates the codes of columns
// (8P + 2d, 8P + 2d + 1) in the low and high half-word, ready to be turned into a pair of fp16 values.
//   4-bit (P = 0..3): bits 16h + 4P .. +3 of dword d.
//   2-bit (P = 0..7): the dword is read as 8 nibbles; nibble nn = (P % 4) + 4h holds
//       for P < 4 (the first 32 columns of the unit) the code in nibble bits 1 (code bit 0) and 2 (code bit 1);
//       for P >= 4 (the last 32 columns) code bit 0 in nibble bit 3 and code bit 1 in bit 0 of nibble
//       (nn + 1) % 8 of the same dword, i.e. in dword bits 4nn + 3 and (4nn + 4) % 32.
//     Reason: bits 1, 2 of a nibble are the two exponent bits of an fp4 (E2M1) number with sign and
//     mantissa bit cleared, so dword & 0x22222222 / 0x44444444 / 0x66666666 ARE eight fp4 numbers
//     1.0 * bit0 / 2.0 * bit1 / {0, 1, 2, 4}[code], the B operand of v_mfma_f32_16x16x128_f8f6f4, with no
//     unpacking; the same three masks on the dword rotated right by 2 give the last 32 columns.  The
//     per-weight decode reads the same layout as fields at bit offsets 1, 3, 5, 7 of the half-words of
//     the dword and of the dword rotated right by 8.
//
// Side part of a tile record for meta = MPQ_META_PAPER (Sec. 3.3 "Memory Alignment"; g1 = 16), every
// array 16-byte aligned, each followed by one all-zero entry that padding pieces point at:
//         meta1a  (T3+1) x 16 x 2 B    per (triple of consecutive 2-bit stream groups, row) one 16-bit word:
//                                      bits 0-1, 2-3, 4-5 the three zero points, bits 6-9 the first scale (4 bits),
//                                      bits 10-12 and 13-15 the second and third scale (3 bits each); T3 = ceil(n2 / 3)
//         meta1b  (n4+1) x 16 x 1 B    per (4-bit stream group, row): scale in bits 0-3, zero point in bits 4-7
//         s2      E x 2 B, z2  E x 1 B the fp16 second-order scales and the byte-padded second-order zeros, E
//                                      entries indexed like meta2 above: (S+1) x 16 (g2_axis 0) or (G+1) x nsub
//         outl    as above
//   unit table word 1 of a piece: bits 0-15 = byte offset of its triple inside meta1a, with the position of
//   the group in the triple (0..2) in bits 0-1 (2-bit piece), or byte offset of its group inside meta1b (4-bit
//   piece); bits 16-31 = index of its first second-order entry (the lane adds its row, or its block of rows).
//
// Sections and tile records start on 256-byte boundaries; padding bytes are zero.
#ifndef MPQ_FORMAT_H_
#define MPQ_FORMAT_H_

#include <stdint.h>

#define MPQ_MAGIC 0x3151504Du /* "MPQ1" */
#define MPQ_VERSION 9u
#define MPQ_TILE_ROWS 16
#define MPQ_UNITS_PER_BLOCK 4
#define MPQ_BLOCK_BYTES 1024
#define MPQ_SECTION_ALIGN 256
#define MPQ_OTILE_HEAD 128 /* bytes of the row-start table at the head of a tile's outlier record */

typedef struct {
  uint32_t magic, version;
  int32_t N, K, g1, g2, g2_axis;
  int32_t G, S, n2, n4;
  int32_t U2, U4;  /* 16-byte units per row in the 2-bit / 4-bit stream */
  int32_t B2, B4;  /* blocks (4 units x 16 rows) per row tile in each stream */
  int32_t T;       /* row tiles */
  int64_t nnz;
  uint64_t off_units, off_tiles;
  uint64_t tile_stride; /* bytes from one tile record to the next */
  uint64_t side_bytes;  /* meta1 + meta2 + outlier record of a tile */
  uint64_t codes_off;   /* offset of the code blocks inside a tile record */
  uint64_t ocap;        /* words per tile in the outlier records (multiple of 32) */
  uint64_t meta;        /* MPQ_META_BYTES or MPQ_META_PAPER */
  uint64_t oidx_off;    /* offset of the outlier block index inside a tile record; 0 = the blob has none */
  uint64_t total_bytes;
  /* bit g = K-group g holds 4-bit codes (all zero if G > MPQ_IS4_BITS: the header then does not say
     which groups are 4-bit).  With it a unit's table entry follows from the header alone, so the host
     can hand entries to a kernel as arguments instead of the kernel loading them. */
  uint8_t is4_bits[256 - 4 * 16 - 8 - 8 * 8 - 8];
} MpqHeader;
#define MPQ_IS4_BITS (8 * (256 - 4 * 16 - 8 - 8 * 8 - 8))

/* pieces (groups) per 2-bit / 4-bit unit, entries of meta2 per group for g2_axis 1, bytes of meta2 */
static inline int32_t mpq_pu2(int32_t g1) { return g1 >= 64 ? 1 : 64 / g1; }
static inline int32_t mpq_pu4(int32_t g1) { return g1 >= 32 ? 1 : 32 / g1; }
static inline int32_t mpq_nsub(int32_t g2) { return g2 >= MPQ_TILE_ROWS ? 1 : MPQ_TILE_ROWS / g2; }
static inline uint64_t mpq_meta2_bytes(const MpqHeader* h) {
  return h->g2_axis == 0 ? 64ull * ((uint64_t)h->S + 1)
                         : (4ull * (uint64_t)mpq_nsub(h->g2) * ((uint64_t)h->G + 1) + 15ull) / 16ull * 16ull;
}
/* offset of the all-zero entry of meta2 (what padding pieces point at) */
static inline uint32_t mpq_meta2_zero(const MpqHeader* h) {
  return h->g2_axis == 0 ? 64u * (uint32_t)h->S : 4u * (uint32_t)mpq_nsub(h->g2) * (uint32_t)h->G;
}
/* meta = MPQ_META_PAPER: second-order entries per tile (the last MPQ_TILE_ROWS or nsub of them are the zero
 * entries), triples of 2-bit groups, and the byte offsets of the four arrays inside the side part */
static inline uint32_t mpq_p_entries(const MpqHeader* h) {
  return h->g2_axis == 0 ? 16u * ((uint32_t)h->S + 1) : (uint32_t)mpq_nsub(h->g2) * ((uint32_t)h->G + 1);
}
static inline uint32_t mpq_p_zero_entry(const MpqHeader* h) {
  return h->g2_axis == 0 ? 16u * (uint32_t)h->S : (uint32_t)mpq_nsub(h->g2) * (uint32_t)h->G;
}
static inline uint32_t mpq_p_triples(const MpqHeader* h) { return ((uint32_t)h->n2 + 2u) / 3u; }
static inline uint32_t mpq_p_off_m1b(const MpqHeader* h) { return 32u * (mpq_p_triples(h) + 1u); }
static inline uint32_t mpq_p_off_s2(const MpqHeader* h) { return mpq_p_off_m1b(h) + 16u * ((uint32_t)h->n4 + 1u); }
static inline uint32_t mpq_p_off_z2(const MpqHeader* h) { return mpq_p_off_s2(h) + ((2u * mpq_p_entries(h) + 15u) & ~15u); }
static inline uint32_t mpq_p_off_outl(const MpqHeader* h) { return mpq_p_off_z2(h) + ((mpq_p_entries(h) + 15u) & ~15u); }

#ifdef __cplusplus
static_assert(sizeof(MpqHeader) == 256, "header must be 256 bytes");
#include "../../include/mpq.h"
// (The two functions below are shared by the library's two source files and are not exported.)
// Accepts a header only if it is byte for byte what the packer writes for the shape it records
// (the bitmap of 4-bit groups must have n4 bits set, none at or beyond G).
__attribute__((visibility("hidden"))) mpq_status mpq_internal_check_header(const void* hdr_host, MpqHeader* out);
// Word 1 (meta1 offset | meta2 offset << 16) of the table entries of the 4 * (B2 + B4) units, from the
// header alone; false if the header carries no bitmap or a unit holds several groups (g1 < 64).
__attribute__((visibility("hidden"))) bool mpq_internal_unit_words(const MpqHeader* h, uint32_t* words);
#endif

#endif /* MPQ_FORMAT_H_ */
