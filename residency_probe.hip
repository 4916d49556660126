// residency_probe.hip - how many workgroups a compute unit of the GPU holds at once, against static LDS size,
// waves per workgroup and live vector registers per lane.  Stand-alone (no part of the library):
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 residency_probe.hip -o residency_probe && ./residency_probe
//
// Every workgroup reads the 100 MHz wall clock when it starts, touches its LDS and holds its place for 4 us
// (a bounded wait); 2048 workgroups are launched, and those that started within 3 us of the first were
// resident together.  The library's LDS size classes and register budgets follow from the table it prints.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                      \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      printf("%s failed: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__);    \
      exit(1);                                                                     \
    }                                                                              \
  } while (0)

constexpr int GRID = 2048;

// NV live vector registers per lane (0: none beyond what the loop needs), LDSB bytes of static LDS
template <int LDSB, int NV>
__global__ void __launch_bounds__(1024) hold(unsigned long long* out, const int hold_ticks, const float* src) {
  __shared__ unsigned char lds[LDSB];
  const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
  float v[NV > 0 ? NV : 1];
#pragma unroll
  for (int k = 0; k < NV; ++k) v[k] = src[threadIdx.x + 64 * k];
  lds[threadIdx.x] = (unsigned char)threadIdx.x;
  __syncthreads();
  unsigned long long t = t0;
  for (int it = 0; it < 100000 && t - t0 < (unsigned long long)hold_ticks; ++it) {  // at most hold_ticks / 100 us
    __builtin_amdgcn_s_sleep(8);
#pragma unroll
    for (int k = 0; k < NV; ++k) v[k] = v[k] * 1.0001f + v[(k + 1) % (NV > 0 ? NV : 1)];
    t = __builtin_amdgcn_s_memrealtime();
  }
  float s = 0;
#pragma unroll
  for (int k = 0; k < NV; ++k) s += v[k];
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x] = t0;
    out[2 * blockIdx.x + 1] = lds[5] + (unsigned long long)s;
  }
}

template <int LDSB, int NV>
static void run(const int waves, const int cus, unsigned long long* dev, std::vector<unsigned long long>& host, const float* src) {
  CK(hipMemset(dev, 0, GRID * 16));
  hipLaunchKernelGGL((hold<LDSB, NV>), dim3(GRID), dim3(waves * 64), 0, 0, dev, 400, src);
  CK(hipGetLastError());
  CK(hipDeviceSynchronize());
  CK(hipMemcpy(host.data(), dev, GRID * 16, hipMemcpyDeviceToHost));
  unsigned long long first = ~0ull;
  for (int g = 0; g < GRID; ++g) first = std::min(first, host[2 * g]);
  int early = 0;
  for (int g = 0; g < GRID; ++g) early += host[2 * g] - first < 300;
  hipFuncAttributes fa;
  CK(hipFuncGetAttributes(&fa, (const void*)hold<LDSB, NV>));
  printf("LDS %6d B, %3d registers per lane, %2d waves: %4d of %d workgroups at once = %.2f per compute unit = %.1f waves per SIMD\n",
         LDSB, fa.numRegs, waves, early, GRID, early / (double)cus, early / (double)cus * waves / 4.0);
  fflush(stdout);
}

int main() {
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  printf("# %s, %d compute units\n", prop.name, cus);
  unsigned long long* dev;
  float* src;
  CK(hipMalloc(&dev, GRID * 16));
  CK(hipMalloc(&src, (1024 + 64 * 100) * 4));
  CK(hipMemset(src, 0, (1024 + 64 * 100) * 4));
  std::vector<unsigned long long> host(GRID * 2);
  for (int waves : {4, 8, 16}) {
    run<1024, 0>(waves, cus, dev, host, src);
    run<16 * 1024, 0>(waves, cus, dev, host, src);
    run<20 * 1024, 0>(waves, cus, dev, host, src);
    run<30 * 1024, 0>(waves, cus, dev, host, src);
    run<32 * 1024, 0>(waves, cus, dev, host, src);
    run<36 * 1024, 0>(waves, cus, dev, host, src);
    run<40 * 1024, 0>(waves, cus, dev, host, src);
    run<41 * 1024, 0>(waves, cus, dev, host, src);
    run<48 * 1024, 0>(waves, cus, dev, host, src);
    run<52 * 1024, 0>(waves, cus, dev, host, src);
    run<53 * 1024, 0>(waves, cus, dev, host, src);
    run<64 * 1024, 0>(waves, cus, dev, host, src);
    run<80 * 1024, 0>(waves, cus, dev, host, src);
    run<160 * 1024, 0>(waves, cus, dev, host, src);
  }
  for (int waves : {8, 16}) {
    run<32 * 1024, 36>(waves, cus, dev, host, src);
    run<32 * 1024, 44>(waves, cus, dev, host, src);
    run<32 * 1024, 52>(waves, cus, dev, host, src);
    run<32 * 1024, 60>(waves, cus, dev, host, src);
    run<32 * 1024, 76>(waves, cus, dev, host, src);
    run<32 * 1024, 100>(waves, cus, dev, host, src);
  }
  return 0;
}
