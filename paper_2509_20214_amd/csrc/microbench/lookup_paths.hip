// Micro-benchmark behind the statement that the V = 1 trellis is bound by its LDS gather and that sending part
// of the lookups through the vector memory path does not help: random 16-bit-state lookups in an fp16 table,
// through LDS only, through vector memory only (table in L2, or small enough for L1), and through both pipes
// together in several proportions.  Stand-alone program (no part of libqp.so): bench.py --micro builds and runs it.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// per iteration: NL lookups through LDS and NG through global memory, all independent; indices from an LCG
template <int NL, int NG, int TABKB>
__global__ __launch_bounds__(1024) void k_mix(const uint16_t* __restrict__ gtab, uint32_t* out, int iters, uint32_t seed) {
  extern __shared__ uint8_t lds[];
  if (NL > 0) {
    const u32x4* g4 = (const u32x4*)gtab; u32x4* l4 = (u32x4*)lds;
    for (int i = threadIdx.x; i < TABKB * 64; i += blockDim.x) l4[i] = g4[i];
    __syncthreads();
  }
  uint32_t s = seed ^ (threadIdx.x * 747796405u + blockIdx.x * 2891336453u);
  uint32_t acc = 0;
  const uint32_t mask = TABKB * 1024 - 2;
  for (int it = 0; it < iters; ++it) {
    uint32_t idxl[NL > 0 ? NL : 1], idxg[NG > 0 ? NG : 1];
#pragma unroll
    for (int u = 0; u < NL; ++u) { s = s * 1664525u + 1013904223u; idxl[u] = (s >> 7) & mask; }
#pragma unroll
    for (int u = 0; u < NG; ++u) { s = s * 1664525u + 1013904223u; idxg[u] = (s >> 7) & mask; }
    uint16_t vl[NL > 0 ? NL : 1], vg[NG > 0 ? NG : 1];
#pragma unroll
    for (int u = 0; u < NG; ++u) vg[u] = *(const uint16_t*)((const uint8_t*)gtab + idxg[u]);
#pragma unroll
    for (int u = 0; u < NL; ++u) vl[u] = *(const uint16_t*)(lds + idxl[u]);
#pragma unroll
    for (int u = 0; u < NL; ++u) acc += vl[u];
#pragma unroll
    for (int u = 0; u < NG; ++u) acc += vg[u];
  }
  if (acc == 0x12345678u) out[0] = acc;
}

int main() {
  hipDeviceProp_t pr; CK(hipGetDeviceProperties(&pr, 0));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  uint16_t* tab; CK(hipMalloc(&tab, 1 << 20)); CK(hipMemset(tab, 1, 1 << 20));
  uint32_t* out; CK(hipMalloc(&out, 4096));
  const int grid = 256, iters = 400;
  const double clk = 2.4e9;
  auto run = [&](const char* name, auto kern, int lds_bytes, int per_iter) {
    CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(1024), lds_bytes, 0, tab, out, iters, 1u); CK(hipDeviceSynchronize());
    float best = 1e9;
    for (int r = 0; r < 3; ++r) {
      CK(hipEventRecord(e0)); hipLaunchKernelGGL(kern, dim3(grid), dim3(1024), lds_bytes, 0, tab, out, iters, 1u);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (ms < best) best = ms;
    }
    double lookups = (double)1024 * iters * per_iter;   // per CU
    printf("%-44s %8.3f ms  %6.2f lookups/clk/CU  (%5.2f clk per wave-instruction)\n", name, best, lookups / (best * 1e-3 * clk), 64.0 * best * 1e-3 * clk / lookups);
  };
  run("LDS 8 / global 0, 128 KiB table", k_mix<8, 0, 128>, 131072, 8);
  run("LDS 0 / global 8, 128 KiB table (L2)", k_mix<0, 8, 128>, 0, 8);
  run("LDS 0 / global 8, 16 KiB table (L1)", k_mix<0, 8, 16>, 0, 8);
  run("LDS 0 / global 8, 4 KiB table (L1)", k_mix<0, 8, 4>, 0, 8);
  run("LDS 7 / global 1, 128 KiB", k_mix<7, 1, 128>, 131072, 8);
  run("LDS 6 / global 2, 128 KiB", k_mix<6, 2, 128>, 131072, 8);
  run("LDS 8 / global 1 (9 per iteration), 128 KiB", k_mix<8, 1, 128>, 131072, 9);
  run("LDS 8 / global 2 (10 per iteration), 128 KiB", k_mix<8, 2, 128>, 131072, 10);
  printf("done\n");
  return 0;
}
