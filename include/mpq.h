/*
 * mpq.h - C ABI of the 2/4/16-bit mixed-precision weight library for MI355X (gfx950).
 *
 * The library implements the decode-time hot path of arXiv 2311.16442 ("Fast and Efficient 2-bit
 * LLM Inference on GPU: 2/4/16-bit in a Weight Matrix with Asynchronous Dequantization"):
 * y = W x (and Y = X W^T for a small batch) where W is stored as
 *   - per-K-group 2-bit or 4-bit integer codes (Sec. 3.3 "Intra-weight Quantization": the bit width
 *     is chosen per group of g1 input channels and is the same for every output channel),
 *   - a quantized first-order scale and an integer first-order zero point per (row, group), the
 *     scale being recovered by a second-order dequantization with an fp16 (scale, zero) pair
 *     (Sec. 2.2 eq. 5; Sec. 3.3; Algorithm 1, second-order dequantization step),
 *   - fp16 outliers in CSR form, one 32-bit word (fp16 value, 16-bit column) per outlier plus one
 *     32-bit running count per row, located only inside 2-bit groups (Sec. 2.3, Sec. 4.3).
 *
 * Conventions.  W is N x K (N output channels = rows, K input channels = columns).  g1 = first
 * order group size along K, G = K/g1 groups per row, g2 = first-order groups per second-order
 * pair, S = ceil(G/g2).  All fp16 values cross this boundary as their 16-bit patterns (uint16_t).
 *
 * What one weight decodes to (all arithmetic IEEE, round-to-nearest-even, no fused operations):
 *   s1        = fp16( (fp32(s_int) - fp32(z2)) * fp32(s2) )          second-order dequantization
 *   Wd[n][k]  = fp16( fp32(code - z1) * fp32(s1) )                   first-order dequantization
 *   Wfull     = fp16( fp32(Wd) + fp32(val) ) at outlier positions    outliers are additive
 *   y[n]      = sum_k Wd[n][k] x[k] + sum_{outliers of row n} val x[col]
 *
 * Memory.  The library never allocates, frees or retains device memory and keeps no state between
 * calls (mpq_gemm_static alone remembers, per device, the address of the library's own scratch array):
 * every choice a call makes follows from its arguments and from the compute-unit count of the
 * current device, which is queried in the call (MPQ_ERR_HIP if the query fails).  Host entry points take HOST pointers; device entry points take DEVICE pointers for bulk
 * data and a HOST pointer to the blob header (the first MPQ_HEADER_BYTES bytes of the packed
 * blob), so that no call ever needs a device-to-host copy.  All pointers are owned by the caller.
 * Device entry points only enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 * default stream) and return without waiting for it.
 *
 * Errors.  Every entry point returns an mpq_status; nothing is launched unless all arguments
 * validate.  No entry point throws or aborts.  MPQ_ERR_HIP reports the status of the call's own
 * launches only, taken from the launch calls' return values: the thread's HIP last-error state is neither
 * read nor cleared, so an error an earlier HIP call of the caller left pending is not reported and stays pending;
 * after MPQ_ERR_HIP the output buffer is undefined, since an entry point that needs two kernels may
 * have enqueued the first.
 */
#ifndef MPQ_H_
#define MPQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MPQ_HEADER_BYTES 256u
#define MPQ_MAX_M 32          /* largest batch the small-M product accepts */
#define MPQ_MAX_MULTI 8       /* most products one mpq_gemv_multi call accepts */
#define MPQ_STATIC_SCRATCH_BYTES (32u << 20) /* device scratch inside the library that mpq_gemm_static uses */

typedef enum {
  MPQ_OK = 0,
  MPQ_ERR_NULL = 1,            /* a required pointer is NULL */
  MPQ_ERR_SHAPE = 2,           /* N, K, g1, g2, M outside what the format allows */
  MPQ_ERR_ALIGN = 3,           /* a device pointer is not 16-byte aligned */
  MPQ_ERR_CODE_RANGE = 4,      /* a code exceeds 2^b - 1 for its group's bit width b */
  MPQ_ERR_OUTLIER_IN_4BIT = 5, /* an outlier column lies in a 4-bit group (Sec. 4.3 forbids it) */
  MPQ_ERR_CSR = 6,             /* row_ptr not monotone / columns not strictly increasing / col >= K */
  MPQ_ERR_BLOB = 7,            /* header magic, version or recorded sizes do not match */
  MPQ_ERR_SIZE = 8,            /* caller's buffer is smaller than required */
  MPQ_ERR_UNSUPPORTED = 9,     /* valid format that this build's kernels do not implement */
  MPQ_ERR_HIP = 10             /* the HIP runtime reported a launch error */
} mpq_status;

/* Shape of a matrix in the logical format. g1 must be 16, 32, 64 or 128 (MPQ_ERR_UNSUPPORTED
 * otherwise). g2_axis: 0 = a second-order pair covers g2 consecutive groups along K of one row (what
 * the benchmark configurations state); 1 = it covers the same K-group of g2 consecutive rows (the
 * paper's "direction of output channels", Sec. 2.2), with g2 a divisor or a multiple of 16. */
typedef struct {
  int32_t N, K, g1, g2, g2_axis;
  int32_t meta;  /* how scales and zero points are stored, see MPQ_META_* (0 if left out of an initialiser) */
} mpq_desc;

/* meta = MPQ_META_BYTES: s_int and z1 one byte each per (row, group), (s2, z2) two fp16 values: what the
 * benchmark configurations state.
 * meta = MPQ_META_PAPER: the paper's aligned packing (Sec. 3.3 "Memory Alignment"), for g1 = 16:
 *   - the three 2-bit zero points and the three scales of three consecutive 2-bit groups of a row share
 *     ONE 16-bit word: the first scale has Ns = 4 bits, the other two are held in 3 bits ("Scale
 *     Clipping"; which two, and how, the paper does not say: here the second and third group of every
 *     triple of 2-bit groups, counted in K order over the 2-bit groups of the row, must have s_int <= 7 -
 *     a quantizer clips them - and the first s_int <= 15);
 *   - a 4-bit group has a 4-bit scale and a 4-bit zero point in one byte (the paper's bit count
 *     charges 4-bit groups nothing for these; they are stored and counted here);
 *   - the second-order zero is an Ns-bit integer padded to a byte ("Zero Padding"), next to the fp16
 *     second-order scale: z2 must be the fp16 pattern of an integer 0..15.
 * The logical arrays keep their shapes and the decode formula is the one at the top of this file; the
 * packer refuses values outside these ranges with MPQ_ERR_CODE_RANGE. */
#define MPQ_META_BYTES 0
#define MPQ_META_PAPER 1

/* Logical (unpacked) matrix: what a quantizer hands to mpq_pack_host. HOST pointers, read-only. */
typedef struct {
  const uint8_t* is4;      /* [G]     1 = the group is 4-bit for all rows, 0 = 2-bit            */
  const uint8_t* codes;    /* [N*K]   one code per byte, row-major                               */
  const uint8_t* s_int;    /* [N*G]   quantized first-order scale                                */
  const uint8_t* z1;       /* [N*G]   first-order zero point                                     */
  const uint16_t* s2;      /* [N*S]   fp16 second-order scale (g2_axis 0), else [ceil(N/g2)*G]   */
  const uint16_t* z2;      /* same shape, fp16 second-order zero                                 */
  const int32_t* row_ptr;  /* [N+1]   CSR row pointer, row_ptr[0] = 0                            */
  const uint16_t* col;     /* [nnz]   column index, strictly increasing inside a row             */
  const uint16_t* val;     /* [nnz]   fp16 outlier value                                         */
} mpq_logical;

/* The arrays of mpq_logical as outputs (HOST, caller-allocated, same shapes; col / val hold
 * `outlier_capacity` entries). */
typedef struct {
  uint8_t* is4;
  uint8_t* codes;
  uint8_t* s_int;
  uint8_t* z1;
  uint16_t* s2;
  uint16_t* z2;
  int32_t* row_ptr;
  uint16_t* col;
  uint16_t* val;
} mpq_logical_out;

/* Human-readable name of a status code; never NULL. */
const char* mpq_status_str(mpq_status s);

/* Average stored bits per weight.
 * mode 0: bits actually stored by this format without alignment padding:
 *         8 * (codes + 2 B per (row,group) + 4 B per (row,super-group) + 4 B per outlier
 *              + 4 B per row pointer) / (N*K); for d->meta = MPQ_META_PAPER the metadata terms are
 *         2 B per (row, triple of 2-bit groups), 1 B per (row, 4-bit group), 3 B per second-order pair.
 * mode 1: the paper's mixed-precision formula (Sec. 3.3, the display after "the average bit-width
 *         of each weight element"): alpha*(2 + (2+Ns)/g1 + (Ns+16)/(g1*g2)) + (1-alpha)*4 with
 *         alpha = 1 - n4/G and Ns = `ns_bits`, plus the outlier increment (16+16-2)*nnz/(N*K)
 *         (Sec. 4.2).
 * mode 2: the same with the paper's aligned storage of the metadata (Sec. 3.3 "Memory Alignment") in
 *         place of the ideal counts: one 16-bit word for the zero points and scales of three 2-bit
 *         groups (16/(3 g1) bits per weight instead of (2+Ns)/g1) and the second-order zero padded
 *         to whole bytes.  An accounting only: this library stores uint8 scales and zero points
 *         (mode 0).
 * Returns a negative value on invalid arguments. */
double mpq_avg_bits(const mpq_desc* d, int32_t n4, int64_t nnz, int mode, int ns_bits);

/* Reference quantizer: float weights W[N*K] (row-major, HOST) -> the logical format.
 *   - Sec. 3.3 (eq. 9 with the Hessian term set to one: no calibration data): the n4 groups of input
 *     channels with the largest sum of squared weights over all rows become 4-bit (ties: lower index);
 *   - Sec. 4.3: per row the round(p_o * number of 2-bit columns) weights of largest magnitude among
 *     the row's 2-bit columns are outliers (ties: lower column); they do not widen their group's
 *     range, and their stored value is fp16(w - dequantized dense value) (dense + sparse, Sec. 2.3);
 *   - Sec. 2.2 eqs. 2-4 per (row, group) over the non-outlier weights: s = (max - min) / (2^N - 1)
 *     (a constant group: s = |w|, or 1), z = clamp(round(-min / s), 0, 2^N - 1),
 *     code = clamp(round(w / s) + z, 0, 2^N - 1);
 *   - second-order quantization of the scales to 8 bits along d->g2_axis in groups of g2:
 *     s2 = fp16(max((s_max - s_min) / 255, s_max / 2047)) (the second term keeps |z2| <= 2047, which
 *     fp16 holds exactly, when the scales are nearly equal), z2 = fp16(round(-s_min / s2)),
 *     s_int = clamp(round(s / s2) + z2, 0, 255); zero points and codes are then computed against the
 *     scale as the decoder reconstructs it, fp16((s_int - z2) * s2).
 * All arithmetic in binary64, round() = round half to even, fp16 conversions through binary32.
 * `*nnz` receives the number of outliers; MPQ_ERR_SIZE if it exceeds `outlier_capacity`
 * (N * round(p_o * (G - n4) * g1) entries are needed).  MPQ_ERR_SHAPE for n4 outside [0, G] or
 * p_o outside [0, 1]. */
mpq_status mpq_quantize_host(const mpq_desc* d, const float* W, int32_t n4, double p_o,
                             const mpq_logical_out* out, int64_t outlier_capacity, int64_t* nnz);

/* Entries the col / val arrays of mpq_quantize_host must hold for these arguments:
 * N * round(p_o * (G - n4) * g1) (Sec. 4.3: a fixed share of every row's 2-bit columns). */
mpq_status mpq_quantize_outlier_capacity(const mpq_desc* d, int32_t n4, double p_o, int64_t* capacity);

/* Size in bytes of the packed blob for this shape, 4-bit map and outlier row pointer.
 * `is4` is a HOST array of G bytes, `row_ptr` a HOST array of N+1 entries (the blob stores the
 * outliers of every 16-row tile in a record padded to the fullest tile). */
mpq_status mpq_packed_size(const mpq_desc* d, const uint8_t* is4, const int32_t* row_ptr, size_t* bytes);

/* Sec. 3.3 "Memory Alignment": split the codes into a 2-bit stream and a 4-bit stream whose
 * per-lane units are 16 bytes, homogeneous in bit width and 16-byte aligned, interleave the
 * per-group (s_int, z1) bytes and the (s2, z2) halves, and store the outliers as 32-bit words
 * (fp16 value, 16-bit column) with a 32-bit running count per row (Sec. 2.3), grouped by row tile.
 * Validates the logical matrix completely (code ranges, CSR order, outliers only in 2-bit groups)
 * before writing.  `blob_host` must hold `bytes` >= mpq_packed_size(...) bytes; all of them are
 * written (padding is zero).  The blob is position independent and may be copied byte for byte. */
mpq_status mpq_pack_host(const mpq_desc* d, const mpq_logical* w, void* blob_host, size_t bytes);

/* Read back the shape recorded in a blob header (HOST pointer to at least MPQ_HEADER_BYTES). */
mpq_status mpq_blob_info(const void* hdr_host, mpq_desc* out, int64_t* nnz, int32_t* n4,
                         uint64_t* total_bytes);

/* Where the rows live in a blob: `count` records of `record_bytes` bytes, the first at byte
 * `first_offset`, record t holding everything of rows 16 t .. 16 t + 15 (codes, scale words, outliers)
 * and nothing else.  Records can be copied, reordered or dealt to several blobs with the same header
 * fields (Sec. 3.3: the bit width of a group is the same for every row, so rows shard freely): a blob
 * whose records are those of another in a different order is that matrix with its 16-row blocks in that
 * order (if N is a multiple of 16). */
mpq_status mpq_blob_tiles(const void* hdr_host, uint64_t* first_offset, uint64_t* record_bytes, int32_t* count);

/* Dequantize the whole matrix to row-major fp16 W_out[N*K] (device), bit-exact to the definition
 * at the top of this file (eq. 5 applied twice).  add_outliers != 0 adds the CSR values. */
mpq_status mpq_dequant(const void* hdr_host, const void* blob_dev, uint16_t* W_out_dev,
                       int add_outliers, void* stream);

/* Algorithm 1 (GEMV with asynchronous dequantization) with the outlier product of Sec. 4.3 fused
 * in: y[n] = fp16( sum_k Wd[n][k] x[k] + sum_j val_j x[col_j] ), fp32 accumulation.
 * x_dev: K fp16 values, y_dev: N fp16 values (overwritten), both 16-byte aligned, not aliased.
 * The kernels stage a tile's scale words and outlier words (4 bytes per outlier, the fullest 16-row tile of the
 * matrix counts) in on-chip memory next to the activations: a matrix whose fullest tile does not fit there -
 * tens of thousands of outliers in 16 rows, far beyond the 0.2-0.5 % of Sec. 4.3 - is MPQ_ERR_UNSUPPORTED in
 * mpq_gemv and the batch products (nothing is launched); mpq_dequant has no such limit. */
mpq_status mpq_gemv(const void* hdr_host, const void* blob_dev, const uint16_t* x_dev,
                    uint16_t* y_dev, void* stream);

/* `count` independent matrix-vector products (1 <= count <= MPQ_MAX_MULTI) in ONE kernel launch:
 * y_p = W_p x_p for every p, each exactly as mpq_gemv defines it (Algorithm 1, Sec. 4.3).  For
 * products that do not depend on each other - separate projections of a layer, the experts a token
 * is routed to - this saves the fixed cost of a launch per product.  The four arrays are HOST
 * arrays of `count` entries: header pointers (HOST), blob / x / y pointers (DEVICE).  The matrices
 * may differ in shape but must have the same g1 and the same meta; no y may alias anything else.
 * MPQ_ERR_UNSUPPORTED if the products cannot share one launch configuration. */
mpq_status mpq_gemv_multi(int32_t count, const void* const* hdr_host, const void* const* blob_dev,
                          const uint16_t* const* x_dev, uint16_t* const* y_dev, void* stream);

/* Bytes of device workspace with which mpq_gemm runs its fastest path for this matrix and batch
 * size (0 if it needs none: M = 1, or a batch whose activations fit the on-chip memory next to
 * everything else).  The figure depends on the number of compute units of the current device. */
mpq_status mpq_gemm_workspace_size(const void* hdr_host, int32_t M, size_t* bytes);

/* Small-batch product Y[m][n] = sum_k X[m][k] W[n][k] (+ outliers), 1 <= M <= MPQ_MAX_M.
 * X_dev is M x K row-major fp16, Y_dev is M x N row-major fp16 (overwritten).
 * workspace_dev: caller-owned DEVICE memory of workspace_bytes bytes, 256-byte aligned, that the
 * call may overwrite (partial sums of the kernel for batches whose activations do not fit the
 * on-chip memory); its contents mean nothing before or after the call.  It may be NULL or smaller
 * than mpq_gemm_workspace_size says: the product is then computed by a path that needs none and
 * passes over the weights several times.  The library itself never allocates device memory.  Calls
 * that may run at the same time (different streams) must not share a workspace.
 * M = 1 is mpq_gemv.  Activations must be finite (the batch-1 kernel splits them into fp8 pieces
 * whose sum is exact only for finite values). */
mpq_status mpq_gemm(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev, uint16_t* Y_dev,
                    int32_t M, void* workspace_dev, size_t workspace_bytes, void* stream);

/* A launch plan overrides, for ONE call, choices the library otherwise makes from the shape: it is how
 * tests force every kernel and work split and how sweeps measure them.  0 in a field = the library's
 * own choice; a NULL plan = all zero.  Values a kernel cannot honour (LDS, registers) fall back to the
 * nearest it can, or return MPQ_ERR_UNSUPPORTED where the field says so. */
typedef struct {
  int32_t gemv_path;       /* M = 1: 0 auto, 1 plane-sum kernel (MPQ_ERR_UNSUPPORTED if it cannot run), 2 per-weight decode kernel */
  int32_t gemv_waves;      /* M = 1: waves per workgroup (8 or 16) */
  int32_t gemv_tiles;      /* M = 1: 16-row tiles per workgroup */
  int32_t batch_waves;     /* M > 1, resident-activation kernel: waves per workgroup (4, 8, 16) */
  int32_t max_workgroups;  /* M > 1, resident-activation kernel: cap on its persistent workgroups */
  int32_t large_batch;     /* M > 1: 0 auto, 1 K-range kernel whenever a workspace allows it, -1 never */
  int32_t lb_min_ranges;   /* K-range kernel: least number of ranges */
  int32_t lb_tiles;        /* K-range kernel: tiles per group (1..8) */
  int32_t lb_older16;      /* K-range kernel: sixteenths of a SIMD's blocks for the older of its two waves (1..15) */
  int32_t gemv_older;      /* plane-sum kernel: 1 + the sixteenths of a SIMD's blocks that its oldest wave takes beyond an
                              even share (1 = even split; 0 = the library's choice) */
  int32_t reserved[6];     /* must be 0 */
} mpq_plan;

#define MPQ_KERNEL_GEMV_PLANES 1     /* batch 1, 2-bit groups by plane sums on the fp8/fp4 matrix instruction */
#define MPQ_KERNEL_GEMV_DECODE 2     /* batch 1, every weight decoded */
#define MPQ_KERNEL_BATCH_RESIDENT 3  /* batch with all activations resident on chip */
#define MPQ_KERNEL_BATCH_RANGES 4    /* batch by K ranges through the workspace (two launches) */

/* What a planned call enqueued. */
typedef struct {
  int32_t kernel;               /* MPQ_KERNEL_* of the (last) product kernel */
  int32_t launches;             /* kernel launches enqueued by the call */
  int32_t waves;                /* waves per workgroup */
  int32_t tiles_per_workgroup;  /* M = 1 kernels; tiles per group for the K-range kernel; else 0 */
  int32_t workgroups;
  int32_t reserved[3];
} mpq_report;

/* mpq_gemm under a plan (NULL = none), reporting what ran (report may be NULL).  Same contract as
 * mpq_gemm otherwise; mpq_gemm and mpq_gemv are this call with NULL, NULL. */
mpq_status mpq_gemm_planned(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev, uint16_t* Y_dev,
                            int32_t M, void* workspace_dev, size_t workspace_bytes, void* stream,
                            const mpq_plan* plan, mpq_report* report);

/* mpq_gemm for callers that cannot allocate device memory and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same product, same kernels,
 * same results as mpq_gemm given a workspace of mpq_gemm_workspace_size bytes; the workspace is an
 * array of MPQ_STATIC_SCRATCH_BYTES bytes that is part of the library's device image (every GPU the
 * library runs on holds it until the process ends).  The call allocates and frees nothing.
 * MPQ_ERR_SIZE if this matrix and batch need more than MPQ_STATIC_SCRATCH_BYTES (57344 x 8192 needs
 * 7.6 MiB at M = 16); MPQ_ERR_HIP if the array's address cannot be obtained on the current device (it is
 * asked for on the first call per device and kept - the only state the library holds).
 * All calls on one GPU share the one array: calls that may overlap on a GPU (different streams,
 * different threads) race on it and must be serialised by the caller, or use mpq_gemm with workspaces of
 * their own. */
mpq_status mpq_gemm_static(const void* hdr_host, const void* blob_dev, const uint16_t* X_dev, uint16_t* Y_dev,
                           int32_t M, void* stream);

/* mpq_gemm_workspace_size for a call under `plan` (the number of K ranges is a plan field). */
mpq_status mpq_gemm_workspace_size_planned(const void* hdr_host, int32_t M, const mpq_plan* plan, size_t* bytes);

/* Measurement aid: one launch that reads `bytes` bytes (a multiple of 16 is read) at src_dev once, with
 * 16-byte loads, and does nothing else - the bandwidth the memory system delivers to a kernel of that
 * size, next to which the throughput of the product kernels is reported.  sink_dev may be NULL. */
mpq_status mpq_stream_probe(const void* src_dev, size_t bytes, uint32_t* sink_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MPQ_H_ */
