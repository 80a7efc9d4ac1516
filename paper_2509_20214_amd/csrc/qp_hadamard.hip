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

// Fast path for blocks of 256..16384: thread t holds V consecutive values.  The
// butterfly stages factor over the bits of the element index e = [wave | lane | k]:
// the k bits are done in registers, the lane bits with wavefront shuffles, the wave
// bits after one transpose through LDS (each thread then holds, for V/W positions,
// the W values that differ only in the wave bits).  Stages over different bits commute.
template <int V>
__device__ __forceinline__ void qp_fwht_regs(float (&v)[V], int stride, int count) {
    // in-register butterflies over `count` values spaced `stride` apart, for every offset
#pragma unroll
    for (int h = 1; h < count; h <<= 1)
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const int pos = i / stride;  // index inside its group of `count`
            if ((pos & h) == 0 && pos < count && (i + h * stride) < V) {
                const float a = v[i], b = v[i + h * stride];
                v[i] = a + b;
                v[i + h * stride] = a - b;
            }
        }
}

template <int V>
__global__ __launch_bounds__(1024) void k_hadamard_reg(const half_t *x, const int8_t *signs, int n, int block,
                                                       int64_t ldx, half_t *xr, int64_t ldxr, float norm) {
    extern __shared__ float buf[];
    const int nblk = n / block;
    const int b = blockIdx.x / nblk, q = blockIdx.x - b * nblk;
    const int t = threadIdx.x, lane = t & 63;
    const int T = blockDim.x, W = T >> 6;  // W wavefronts, W <= V (or W == 1)
    const half_t *src = x + (int64_t)b * ldx + (int64_t)q * block + t * V;
    const int8_t *sg = signs + (int64_t)q * block + t * V;
    float v[V];
#pragma unroll
    for (int k = 0; k < V; ++k) v[k] = (float)src[k] * (float)sg[k];
    qp_fwht_regs<V>(v, 1, V);
    const int lane_bits = (T >= 64) ? 6 : 0;
#pragma unroll
    for (int m = 0; m < 6; ++m) {
        if (m < lane_bits) {
            const bool hi = (lane >> m) & 1;
#pragma unroll
            for (int k = 0; k < V; ++k) {
                const float o = __shfl_xor(v[k], 1 << m, 64);
                v[k] = hi ? (o - v[k]) : (v[k] + o);
            }
        }
    }
    half_t *dst = xr + (int64_t)b * ldxr + (int64_t)q * block;
    if (W == 1) {
#pragma unroll
        for (int k = 0; k < V; ++k) dst[t * V + k] = (half_t)(v[k] * norm);
        return;
    }
#pragma unroll
    for (int k = 0; k < V; ++k) buf[t * V + k] = v[k];
    __syncthreads();
    // element (wv, r): wv = wave bits, r in [0, 64 V); this thread takes r = t*(V/W) + qq
    const int per = V / W;      // positions per thread
    const int span = 64 * V;    // elements per wave-bit value
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int qq = i % per, wv = i / per;   // v[i] <-> (wv, r = t*per + qq); i = wv*per + qq
        if (wv < W) v[i] = buf[wv * span + t * per + qq];
    }
    // butterflies over wv: values wv apart sit `per` apart in v[]
#pragma unroll
    for (int h = 1; h < V; h <<= 1) {
        if (h < W) {
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const int wv = i / per;
                if ((wv & h) == 0 && wv + h < W && i + h * per < V) {
                    const float a = v[i], c = v[i + h * per];
                    v[i] = a + c;
                    v[i + h * per] = a - c;
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int qq = i % per, wv = i / per;
        if (wv < W) dst[wv * span + t * per + qq] = (half_t)(v[i] * norm);
    }
}

qp_status qp_launch_hadamard(const void *x, const int8_t *signs, int B, int n, int block, int64_t ldx,
                             void *xr, int64_t ldxr, hipStream_t st) {
    float norm_fast = 1.0f / sqrtf((float)block);
    if (block >= 256 && block <= 16384) {
        const int V = (block <= 1024) ? 4 : (block <= 4096) ? 8 : 16;
        const int threads = block / V, grid = B * (n / block);
        const size_t lds = (threads > 64) ? (size_t)block * sizeof(float) : 0;
        if (V == 4)
            hipLaunchKernelGGL(k_hadamard_reg<4>, dim3(grid), dim3(threads), lds, st, (const half_t *)x, signs, n,
                               block, ldx, (half_t *)xr, ldxr, norm_fast);
        else if (V == 8)
            hipLaunchKernelGGL(k_hadamard_reg<8>, dim3(grid), dim3(threads), lds, st, (const half_t *)x, signs, n,
                               block, ldx, (half_t *)xr, ldxr, norm_fast);
        else
            hipLaunchKernelGGL(k_hadamard_reg<16>, dim3(grid), dim3(threads), lds, st, (const half_t *)x, signs, n,
                               block, ldx, (half_t *)xr, ldxr, norm_fast);
        return qp_check_launch();
    }
    int threads = block / 2;
    if (threads < 64) threads = 64;
    if (threads > 1024) threads = 1024;
    int grid = B * (n / block);
    float norm = 1.0f / sqrtf((float)block);
    hipLaunchKernelGGL(k_hadamard_lds, dim3(grid), dim3(threads), (size_t)block * sizeof(float), st,
                       (const half_t *)x, signs, n, block, ldx, (half_t *)xr, ldxr, norm);
    return qp_check_launch();
}
