// Online rotation of activations (Section 3.3): per block, xr = H (signs .* x) / sqrt(block),
// H the Sylvester Hadamard matrix in natural order, computed as log2(block) butterfly
// stages in fp32 and rounded once to fp16.
#include "qp_internal.h"

// One workgroup per (batch row, block).  The block lives in LDS as fp32; every
// stage h pairs element i with i+h inside groups of 2h.
__global__ __launch_bounds__(1024) void k_hadamard_lds(const half_t *x, const int8_t *signs, int n, int block,
                                                       int64_t ldx, half_t *xr, int64_t ldxr, float norm) {
    extern __shared__ float buf[];
    const int nblk = n / block;
    const int b = blockIdx.x / nblk, q = blockIdx.x - b * nblk;
    const half_t *src = x + (int64_t)b * ldx + (int64_t)q * block;
    const int8_t *sg = signs + (int64_t)q * block;
    for (int i = threadIdx.x; i < block; i += blockDim.x) buf[i] = (float)src[i] * (float)sg[i];
    for (int h = 1; h < block; h <<= 1) {
        __syncthreads();
        for (int p = threadIdx.x; p < block / 2; p += blockDim.x) {
            int i = ((p / h) * 2 * h) + (p % h);
            float u = buf[i], v = buf[i + h];
            buf[i] = u + v;
            buf[i + h] = u - v;
        }
    }
    __syncthreads();
    half_t *dst = xr + (int64_t)b * ldxr + (int64_t)q * block;
    for (int i = threadIdx.x; i < block; i += blockDim.x) dst[i] = (half_t)(buf[i] * norm);
}

qp_status qp_launch_hadamard(const void *x, const int8_t *signs, int B, int n, int block, int64_t ldx,
                             void *xr, int64_t ldxr, hipStream_t st) {
    int threads = block / 2;
    if (threads < 64) threads = 64;
    if (threads > 1024) threads = 1024;
    int grid = B * (n / block);
    float norm = 1.0f / sqrtf((float)block);
    hipLaunchKernelGGL(k_hadamard_lds, dim3(grid), dim3(threads), (size_t)block * sizeof(float), st,
                       (const half_t *)x, signs, n, block, ldx, (half_t *)xr, ldxr, norm);
    return qp_check_launch();
}
