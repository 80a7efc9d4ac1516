// Micro-benchmark behind the choice of the matrix cores at batch 1: issue cost of the multiply of one decode step
// (8 weights per lane) - one v_mfma_f32_16x16x32_f16 against four v_dot2_f32_f16 - alone and behind the step's four
// conflict-free table lookups, with 1, 2 and 4 wavefronts per SIMD.  Stand-alone program (no part of libqp.so):
// bench.py --micro builds and runs it.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int MODE, bool LOOKUP>   // MODE 0: mfma, 1: 4 x dot2
__global__ __launch_bounds__(1024) void k_step(uint32_t* out, int iters, uint32_t seed) {
  __shared__ uint32_t tab[16384];
  for (int i = threadIdx.x; i < 16384; i += blockDim.x) tab[i] = 0x3c003c00u + i;
  __syncthreads();
  uint32_t s = seed + threadIdx.x * 2654435761u;
  u32x4 xw = {0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  float4v acc[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
  float d[4] = {0, 0, 0, 0};
  const uint32_t lane4 = (threadIdx.x & 31) << 2;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      u32x4 a;
      if (LOOKUP) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint32_t ad = ((s >> (5 * c + st)) & 0xff) << 7 | lane4;   // 256 rows x 128 B, conflict-free
          asm volatile("" : "+v"(ad));                                 // four lookups per step in both variants, whatever the compiler can prove
          a[c] = *(const uint32_t*)((const uint8_t*)tab + ad);
        }
        s = s * 1664525u + 1013904223u;
      } else {
        a = u32x4{s, s ^ 0x11u, s + 3, s * 5}; s += 0x01010101u;
      }
      if (MODE == 0) {
        acc[st & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, xw), acc[st & 3], 0, 0, 0);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          d[c] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, a[c]), __builtin_bit_cast(half2v, xw[c]), d[c], false);
      }
    }
  }
  float r = d[0] + d[1] + d[2] + d[3] + acc[0][0] + acc[1][1] + acc[2][2] + acc[3][3];
  if (r == 12345.678f) out[0] = 1;
}

int main() {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  uint32_t* out; CK(hipMalloc(&out, 4096));
  const int iters = 2000;
  auto run = [&](const char* name, auto kern, int threads) {
    hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 0, 0, out, iters, 1u); CK(hipDeviceSynchronize());
    float best = 1e9;
    for (int r = 0; r < 3; ++r) { CK(hipEventRecord(e0)); hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 0, 0, out, iters, 1u);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (ms < best) best = ms; }
    const double steps_per_simd = (double)iters * 8 * (threads / 256);      // wavefronts per SIMD x steps
    printf("%-52s %d wavefront(s) per SIMD: %6.1f clocks per step and SIMD (2.4 GHz)\n", name, threads / 256, best * 1e-3 * 2.4e9 / steps_per_simd);
  };
  for (int t : {256, 512, 1024}) {
    run("multiply only, v_mfma_f32_16x16x32_f16", k_step<0, false>, t);
    run("multiply only, 4 x v_dot2_f32_f16", k_step<1, false>, t);
    run("4 lookups + v_mfma_f32_16x16x32_f16", k_step<0, true>, t);
    run("4 lookups + 4 x v_dot2_f32_f16", k_step<1, true>, t);
  }
  printf("done\n");
  return 0;
}
