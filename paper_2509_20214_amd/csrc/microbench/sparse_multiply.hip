// Micro-benchmark behind the decision NOT to use the structured-sparsity matrix instruction: one decode step's
// lookups (two 8-byte lookups of code pairs per 8 weights, address = shift + and-or) followed by the dense
// v_mfma_f32_16x16x32_f16 per 8 weights, against the same lookups for 16 weights followed by ONE
// v_smfmac_f32_16x16x64_f16 whose dense operand is the 16 weights and whose 2:4-sparse operand stands for the
// activations - with the table of pairs held eight and sixteen times, 1 to 4 wavefronts per SIMD - and the bare
// rate of the two instructions.  Stand-alone program (no part of libqp.so): bench.py --micro builds and runs it.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half16 __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// MODE 0: dense, masks as in the kernel (1 AND per step on average); 1: sparse, half the masks; COPIES 8 or 16
template <int MODE, int LSH>
__global__ __launch_bounds__(1024) void k_step(uint32_t* out, int iters, uint32_t seed) {
  __shared__ uint32_t tab[(1024 << LSH) / 4];
  for (int i = threadIdx.x; i < (1024 << LSH) / 4; i += blockDim.x) tab[i] = 0x3c003c00u + (i & 255);
  __syncthreads();
  uint32_t s = seed + threadIdx.x * 2654435761u;
  u32x4 xw = {0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  uint32_t keep = (threadIdx.x & 16) ? 0xffffffffu : 0u;
  asm volatile("" : "+v"(keep));
  float4v acc[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
  const uint32_t lc = (threadIdx.x & ((1u << (LSH - 3)) - 1)) << 3;
  const int id = (threadIdx.x & 4) ? 0xEEEE : 0x4444;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      u32x4 a;
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        uint32_t t = s >> (10 * c + st);
        uint32_t ad = (t & (1023u << LSH)) | lc;
        asm volatile("" : "+v"(ad));
        u32x2 v = *(const u32x2*)((const uint8_t*)tab + ad);
        a[2 * c] = v[0]; a[2 * c + 1] = v[1];
      }
      s = s * 1664525u + 1013904223u;
      if (MODE == 0) {
        u32x4 m = xw;
        m[st & 3] &= keep;   // one AND per step, as the kernel's 32 per unit
        asm volatile("" : "+v"(m));
        acc[st & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, m), acc[st & 3], 0, 0, 0);
      } else {
        u32x4 a2;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          uint32_t t = s >> (10 * c + st);
          uint32_t ad = (t & (1023u << LSH)) | lc;
          asm volatile("" : "+v"(ad));
          u32x2 v = *(const u32x2*)((const uint8_t*)tab + ad);
          a2[2 * c] = v[0]; a2[2 * c + 1] = v[1];
        }
        s = s * 1664525u + 1013904223u;
        u32x4 m = xw;
        m[st & 3] &= keep;   // one AND per double step
        asm volatile("" : "+v"(m));
        u32x8 w = {a[0], a[1], a[2], a[3], a2[0], a2[1], a2[2], a2[3]};
        acc[st & 3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(half8, m), __builtin_bit_cast(half16, w), acc[st & 3], id, 0, 0);
      }
    }
  }
  float r = acc[0][0] + acc[1][1] + acc[2][2] + acc[3][3];
  if (r == 12345.678f) out[0] = 1;
}

template <int MODE>
__global__ __launch_bounds__(1024) void k_rate(float* out, int iters) {
  half8 a = {1, 2, 3, 4, 5, 6, 7, 8};
  half8 b = {1, 1, 1, 1, 1, 1, 1, 1};
  half16 bb = {1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1};
  float4v acc[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
  const int id = 0x4444 + (threadIdx.x & 1) * 0xaaaa;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (MODE == 0) acc[s & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[s & 3], 0, 0, 0);
      else acc[s & 3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(a, bb, acc[s & 3], id, 0, 0);
    }
  }
  float r = acc[0][0] + acc[1][1] + acc[2][2] + acc[3][3];
  if (r == 12345.678f) out[0] = r;
}

int main() {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  uint32_t* out; CK(hipMalloc(&out, 4096));
  const int iters = 2000;
  auto run = [&](const char* name, auto kern, int threads, int weights_per_it) {
    hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 0, 0, out, iters, 1u); CK(hipDeviceSynchronize());
    float best = 1e9;
    for (int r = 0; r < 3; ++r) { CK(hipEventRecord(e0)); hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 0, 0, out, iters, 1u);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (ms < best) best = ms; }
    const double steps_per_simd = (double)iters * weights_per_it / 8 * (threads / 256);
    printf("%-50s %d wave(s)/SIMD: %6.1f clocks per 8 weights per lane and SIMD (2.4 GHz)\n", name, threads / 256, best * 1e-3 * 2.4e9 / steps_per_simd); fflush(stdout);
  };
  for (int t : {256, 512, 768, 1024}) {
    run("dense mfma, 8 copies", k_step<0, 6>, t, 64);
    run("sparse smfmac, 8 copies", k_step<1, 6>, t, 128);
    run("dense mfma, 16 copies", k_step<0, 7>, t, 64);
    run("sparse smfmac, 16 copies", k_step<1, 7>, t, 128);
  }
  {
    float* outf; CK(hipMalloc(&outf, 64));
    const int it2 = 4000;
    auto rate = [&](const char* name, auto kern, int threads) {
      hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 0, 0, outf, it2); CK(hipDeviceSynchronize());
      float best = 1e9;
      for (int r = 0; r < 3; ++r) { CK(hipEventRecord(e0)); hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 0, 0, outf, it2);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (ms < best) best = ms; }
      printf("%-50s %d wave(s)/SIMD: %6.2f clocks per instruction and SIMD (2.4 GHz)\n", name, threads / 256, best * 1e-3 * 2.4e9 / ((double)it2 * 8 * (threads / 256))); fflush(stdout);
    };
    for (int t : {256, 1024}) { rate("bare v_mfma_f32_16x16x32_f16", k_rate<0>, t); rate("bare v_smfmac_f32_16x16x64_f16", k_rate<1>, t); }
  }
  printf("done\n");
  return 0;
}
