// store_probe.hip - what the write side of the GPU's memory delivers to kernels shaped like the dequantization
// (22016 x 4096 fp16 out = 180 MB, written as 16-row tiles, with 1/8 of that volume read).  Stand-alone:
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 store_probe.hip -o store_probe && ./store_probe
//
// Every kernel writes the whole matrix once; six output buffers (and, where it says so, six input buffers)
// are used in turn so that no launch finds its lines in a cache; time = 30 launches between two events.
//   fill            : every workgroup streams 16-byte words with a grid stride
//   tile R          : a workgroup owns 16 rows, a wave 1 KiB-wide strips of them; one store instruction writes
//                     R rows x 1024/R bytes (R = 16: 64-byte pieces of 16 rows; 8: whole 128-byte lines of 8 rows)
//   wave model D    : four-wave workgroups, 37 KiB of LDS each (four per compute unit); blocks of 16 rows x 512 bytes
//                     dealt round-robin over all waves; per block: 1 KiB loaded D blocks ahead, 160 dependent
//                     multiply-adds, the decoded bytes turned through LDS (8 x 16-byte writes per lane, 8 reads),
//                     eight store instructions of whole lines
//   split D / PART  : 1024 four-wave workgroups; a job = 16 rows x 1 KiB = 16 store instructions of 16 rows x 64 bytes,
//                     i.e. every 128-byte line is written as two halves (or every 64-byte segment as two 32-byte
//                     halves, two segments per row and instruction).  D = lines whose first halves a wave writes
//                     before it writes their second halves (1: the halves follow each other; 8: a job's 8 first
//                     halves, then its 8 second halves; 32: four jobs').  PART = who writes the second halves: the
//                     same wave, the wave next to it in the workgroup, the same wave of a workgroup on the same die
//                     (workgroups go to the eight dies in turn), or of a workgroup on the next die; the two work
//                     through the same jobs in the same order, one half each.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                      \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      printf("%s failed: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__);    \
      exit(1);                                                                     \
    }                                                                              \
  } while (0)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int N = 22016, ROW = 8192;  // rows, bytes per row
constexpr size_t BYTES = (size_t)N * ROW;
constexpr int BLOCKS_PER_TILE = ROW / 512, BLOCKS = (N / 16) * BLOCKS_PER_TILE;

__global__ void __launch_bounds__(256) fill(u32x4* out, const size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const u32x4 v = {(unsigned)i, 1u, 2u, 3u};
    out[i] = v;
  }
}

template <int R, bool NT>
__global__ void __launch_bounds__(256) tile(unsigned char* out) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  constexpr int seg = 1024 / R, lanes_per_row = seg / 16;
  const int r_in = lane / lanes_per_row, col = (lane % lanes_per_row) * 16;
  const size_t row0 = (size_t)blockIdx.x * 16;
  for (int strip = wv; strip < ROW / 1024; strip += 4) {
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const int row = (s * R) % 16 + r_in, cs = ((s * R) / 16) * seg;
      const u32x4 v = {(unsigned)lane, (unsigned)s, (unsigned)strip, (unsigned)blockIdx.x};
      u32x4* p = (u32x4*)(out + (row0 + row) * ROW + (size_t)strip * 1024 + cs + col);
      if (NT) __builtin_nontemporal_store(v, p);
      else *p = v;
    }
  }
}

template <int D>
__global__ void __launch_bounds__(256) wave_model(unsigned char* out, const u32x4* src, const int nwaves, float* sink) {
  __shared__ __align__(16) unsigned char turn[4][64 * 144];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int gw = blockIdx.x * 4 + wv;
  unsigned char* mine = turn[wv];
  float a0 = lane, a1 = lane + 1, a2 = lane + 2, a3 = lane + 3;
  u32x4 q[D];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    const int n = gw + d * nwaves;
    q[d] = src[(size_t)(n < BLOCKS ? n : gw % BLOCKS) * 64 + lane];
  }
  for (int n0 = gw; n0 < BLOCKS; n0 += D * nwaves) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const int n = n0 + d * nwaves;
      if (n >= BLOCKS) break;
      const int t = n / BLOCKS_PER_TILE, c = n - t * BLOCKS_PER_TILE;
      const int ahead = n + D * nwaves < BLOCKS ? n + D * nwaves : n;
#pragma unroll 8
      for (int w = 0; w < 40; ++w) {
        a0 = a0 * 1.0001f + a1; a1 = a1 * 0.9999f + a2; a2 = a2 * 1.0002f + a3; a3 = a3 * 0.9998f + a0;
      }
      const u32x4 v = {(unsigned)__float_as_uint(a0) ^ q[d].x, q[d].y, q[d].z + (unsigned)n, q[d].w};
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        u32x4 w = v;
        w.y += p;
        *(u32x4*)(mine + lane * 144 + p * 16) = w;
      }
      q[d] = src[(size_t)ahead * 64 + lane];
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int pair = (lane >> 3) + s * 8;  // (row, unit): eight lanes write its 128 bytes
        const u32x4 w = *(const u32x4*)(mine + pair * 144 + (lane & 7) * 16);
        *(u32x4*)(out + ((size_t)t * 16 + (pair & 15)) * ROW + (size_t)c * 512 + (pair >> 4) * 128 + (lane & 7) * 16) = w;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
  }
  if (a0 == 12345.678f) sink[0] = a0 + a1 + a2 + a3;
}

constexpr int JOBS = (N / 16) * (ROW / 1024);

// One store instruction: 16 rows x 64 bytes.  PB = 64: half `par` of line l of the job's strip.  PB = 32: the 32-byte
// half `par` of the two 64-byte segments of line l (lanes in pairs).
template <int PB>
__device__ __forceinline__ void store_piece(unsigned char* out, const int job, const int l, const int par, const int lane) {
  const int t = job / (ROW / 1024), strip = job - t * (ROW / 1024);
  const u32x4 v = {(unsigned)lane, (unsigned)l, (unsigned)job, 7u};
  const int at = PB == 64 ? l * 128 + par * 64 + (lane & 3) * 16 : l * 128 + ((lane >> 1) & 1) * 64 + par * 32 + (lane & 1) * 16;
  *(u32x4*)(out + ((size_t)t * 16 + (lane >> 2)) * ROW + (size_t)strip * 1024 + at) = v;
}

template <int D, int PB>
__global__ void __launch_bounds__(256) split_same_wave(unsigned char* out) {
  const int lane = threadIdx.x & 63, gw = blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = gridDim.x * 4;
  constexpr int G = D > 8 ? D / 8 : 1;  // jobs whose halves are interleaved
  for (int base = 0; gw + base * nwaves < JOBS; base += G) {
#pragma unroll
    for (int lg = 0; lg < 8 * G; lg += D) {
#pragma unroll
      for (int par = 0; par < 2; ++par) {
#pragma unroll
        for (int l = lg; l < lg + D; ++l) {
          const int job = gw + (base + l / 8) * nwaves;
          if (job < JOBS) store_piece<PB>(out, job, l % 8, par, lane);
        }
      }
    }
  }
}

// PART 1: the wave next to it in the workgroup; 2: a workgroup on the same die; 3: a workgroup on the next die
template <int PART, int PB>
__global__ void __launch_bounds__(256) split_other(unsigned char* out) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, b = blockIdx.x;
  int par, first, step;
  if (PART == 1) { par = wv & 1; first = b * 2 + (wv >> 1); step = gridDim.x * 2; }
  else if (PART == 2) { par = (b >> 3) & 1; first = ((b & 7) | ((b >> 4) << 3)) * 4 + wv; step = gridDim.x * 2; }
  else { par = b & 1; first = (b >> 1) * 4 + wv; step = gridDim.x * 2; }
  for (int job = first; job < JOBS; job += step) {
#pragma unroll
    for (int l = 0; l < 8; ++l) store_piece<PB>(out, job, l, par, lane);
  }
}

int main() {
  unsigned char* out[6];
  u32x4* src[6];
  float* sink;
  for (int i = 0; i < 6; ++i) {
    CK(hipMalloc(&out[i], BYTES));
    CK(hipMalloc(&src[i], (size_t)BLOCKS * 1024));
    CK(hipMemset(src[i], i + 1, (size_t)BLOCKS * 1024));
  }
  CK(hipMalloc(&sink, 64));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  auto run = [&](const char* name, auto launch) {
    for (int i = 0; i < 6; ++i) launch(i);
    CK(hipGetLastError());
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int r = 0; r < 5; ++r)
      for (int i = 0; i < 6; ++i) launch(i);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    printf("%-58s %7.2f us  %5.2f TB/s written\n", name, ms * 1e3 / 30, BYTES / (ms * 1e-3 / 30) / 1e12);
    fflush(stdout);
  };
  run("fill, 8192 workgroups", [&](int i) { fill<<<8192, 256>>>((u32x4*)out[i], BYTES / 16); });
  run("tile, 16 rows x 64 B per store", [&](int i) { tile<16, false><<<N / 16, 256>>>(out[i]); });
  run("tile, 16 rows x 64 B per store, non-temporal", [&](int i) { tile<16, true><<<N / 16, 256>>>(out[i]); });
  run("tile, 8 rows x 128 B per store", [&](int i) { tile<8, false><<<N / 16, 256>>>(out[i]); });
  run("tile, 8 rows x 128 B per store, non-temporal", [&](int i) { tile<8, true><<<N / 16, 256>>>(out[i]); });
  run("tile, 1 row x 1 KiB per store", [&](int i) { tile<1, false><<<N / 16, 256>>>(out[i]); });
  run("tile, 1 row x 1 KiB per store, non-temporal", [&](int i) { tile<1, true><<<N / 16, 256>>>(out[i]); });
#define MODEL(D, WGS, ONE)                                                                                             \
  run("wave model, " #D " ahead, " #WGS " workgroups, " ONE, [&](int i) {                                              \
    wave_model<D><<<WGS, 256>>>(out[i], src[ONE[0] == 'o' ? 0 : i], (WGS) * 4, sink);                                  \
  });
  MODEL(1, 1024, "one input (cached)")
  MODEL(1, 1024, "six inputs (from memory)")
  MODEL(2, 1024, "six inputs (from memory)")
  MODEL(4, 1024, "six inputs (from memory)")
  MODEL(7, 1024, "six inputs (from memory)")
  MODEL(1, 885, "six inputs (from memory)")
  MODEL(7, 885, "six inputs (from memory)")
  MODEL(7, 768, "six inputs (from memory)")
  MODEL(1, 256, "one input (cached)")
  MODEL(1, 64, "one input (cached)")
#define SPLIT(PB, WHAT)                                                                                                \
  run("split " WHAT ", the two parts follow each other", [&](int i) { split_same_wave<1, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", 2 first parts, then their second parts", [&](int i) { split_same_wave<2, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", 4 first parts, then their second parts", [&](int i) { split_same_wave<4, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", 8 first parts, then their second parts", [&](int i) { split_same_wave<8, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", 16 first parts, then their second parts", [&](int i) { split_same_wave<16, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", 32 first parts, then their second parts", [&](int i) { split_same_wave<32, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", second parts by the next wave of the workgroup", [&](int i) { split_other<1, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", second parts by a workgroup on the same die", [&](int i) { split_other<2, PB><<<1024, 256>>>(out[i]); }); \
  run("split " WHAT ", second parts by a workgroup on the next die", [&](int i) { split_other<3, PB><<<1024, 256>>>(out[i]); });
  SPLIT(64, "128-byte lines into halves")
  SPLIT(32, "64-byte segments into halves")
  return 0;
}
