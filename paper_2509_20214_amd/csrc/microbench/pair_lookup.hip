// Micro-benchmark behind the 2.5-bit vector quantizer's table of code pairs: the lookups of one decode step
// (8 weights per lane) as four 4-byte lookups in a conflict-free table (one per bank and lane; addresses formed
// by two vector operations, or by one SDWA operation as the byte-window decoders do) against two 8-byte lookups
// with a 10-bit index (two neighbouring codes) in a table that is replicated eight or sixteen times only, so that
// lanes do collide - each followed by the step's v_mfma_f32_16x16x32_f16, with 1, 2 and 4 wavefronts per SIMD.
// Stand-alone program (no part of libqp.so): bench.py --micro builds and runs it.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// MODE 0: 4 x b32 conflict-free (256 rows x 128 B); 1: 2 x b64, 8 copies, address (idx << 6) | (lane%8 << 3);
// 2: 2 x b64, 8 copies, 4 slots per 32-byte chunk: (idx>>2)<<8 | (lane%8)<<5 | (idx&3)<<3 ; 3: 2 x b64, 16 copies in 128 KiB: (idx << 7) | (lane%16 << 3)
template <int MODE>
__global__ __launch_bounds__(1024) void k_step(uint32_t* out, int iters, uint32_t seed) {
  __shared__ uint32_t tab[MODE == 3 ? 32768 : 16384];
  for (int i = threadIdx.x; i < (MODE == 3 ? 32768 : 16384); i += blockDim.x) tab[i] = 0x3c003c00u + i;
  __syncthreads();
  uint32_t s = seed + threadIdx.x * 2654435761u;
  u32x4 xw = {0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  float4v acc[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
  const uint32_t lane4 = (threadIdx.x & 31) << 2;
  const uint32_t l8 = (threadIdx.x & 7), l16 = threadIdx.x & 15;
  uint32_t adr[4] = {lane4, lane4, lane4, lane4};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      u32x4 a;
      if (MODE == 4) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int sh = 5 * c + (st & 3) + 1;
          asm volatile("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(adr[c]) : "s"(sh), "v"(s));
          a[c] = *(const uint32_t*)((const uint8_t*)tab + adr[c]);
        }
      } else if (MODE == 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint32_t ad = ((s >> (5 * c + st)) & 0xff) << 7 | lane4;
          asm volatile("" : "+v"(ad));
          a[c] = *(const uint32_t*)((const uint8_t*)tab + ad);
        }
      } else {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          uint32_t idx = (s >> (10 * c + st)) & 1023, ad;
          if (MODE == 1) ad = (idx << 6) | (l8 << 3);
          else if (MODE == 2) ad = ((idx >> 2) << 8) | (l8 << 5) | ((idx & 3) << 3);
          else ad = (idx << 7) | (l16 << 3);
          asm volatile("" : "+v"(ad));
          u32x2 v = *(const u32x2*)((const uint8_t*)tab + ad);
          a[2 * c] = v[0]; a[2 * c + 1] = v[1];
        }
      }
      s = s * 1664525u + 1013904223u;
      acc[st & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, xw), acc[st & 3], 0, 0, 0);
    }
  }
  float r = acc[0][0] + acc[1][1] + acc[2][2] + acc[3][3];
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
    const double steps_per_simd = (double)iters * 8 * (threads / 256);
    printf("%-60s %d wave(s)/SIMD: %6.1f clocks per step and SIMD (2.4 GHz)\n", name, threads / 256, best * 1e-3 * 2.4e9 / steps_per_simd); fflush(stdout);
  };
  for (int t : {256, 512, 1024}) {
    run("4 x b32 conflict-free + mfma", k_step<0>, t);
    run("4 x b32 conflict-free, one SDWA per address + mfma", k_step<4>, t);
    run("2 x b64, 8 copies, (idx<<6)|lane8 + mfma", k_step<1>, t);
    run("2 x b64, 8 copies, 4 slots per chunk + mfma", k_step<2>, t);
    run("2 x b64, 16 copies 128 KiB + mfma", k_step<3>, t);
  }
  printf("done\n");
  return 0;
}
