// Online rotation of activations (Section 3.3): per block, xr = H (signs .* x) / sqrt(block),
// H the Sylvester Hadamard matrix in natural order, computed as log2(block) butterfly
// stages in fp32 and rounded once to fp16.
#include "qp_internal.h"
#include "qp_fwht.h"

// One workgroup per (batch row, block).  The block lives in LDS as fp32; every
// stage h pairs element i with i+h inside groups of 2h.
__global__ __launch_bounds__(1024) void k_hadamard_lds(const half_t *x, const int8_t *signs, int n, int block,
                                                       int64_t ldx, half_t *xr, int64_t ldxr, float norm,
                                                       int pack_bp) {
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
    for (int i = threadIdx.x; i < block; i += blockDim.x)
        xr[qp_xr_index(b, q * block + i, ldxr, pack_bp)] = qp_scale_round(buf[i], norm);
}

template <int V, int W>
__global__ __launch_bounds__(64 * W) void k_hadamard_reg(const half_t *x, const int8_t *signs, int n,
                                                         int64_t ldx, half_t *xr, int64_t ldxr, float norm,
                                                         int pack_bp) {
    constexpr int block = 64 * V * W;
    __shared__ float buf[(W > 1) ? block + block / 32 : 1];
    const int nblk = n / block;
    const int b = blockIdx.x / nblk, q = blockIdx.x - b * nblk;
    const int col0 = q * block;
    qp_fwht_tile<V, W>(true, threadIdx.x, x + (int64_t)b * ldx + col0, signs + col0, norm, buf,
                       [&](int idx, half_t val) { xr[qp_xr_index(b, col0 + idx, ldxr, pack_bp)] = val; });
}

// Blocks of 1024 on the matrix cores: one wavefront per (batch row, block), four per workgroup.
__global__ __launch_bounds__(256) void k_hadamard_1024(const half_t *x, const int8_t *signs, int n, int64_t ldx,
                                                       half_t *xr, int64_t ldxr, int pack_bp, int items) {
    const int lane = threadIdx.x & 63;
    const int it = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (it >= items) return;
    const int nblk = n >> 10;
    const int b = it / nblk, c = it - b * nblk;
    QpHad1024 H;
    H.init(lane);
    const QpHad1024In in = qp_fwht1024_fetch(x + (int64_t)b * ldx + 1024 * c, signs + 1024 * c, lane);
    float4_t o[2][2];
    qp_fwht1024_run(H, in, o);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
            *reinterpret_cast<uint2 *>(xr + qp_xr_index(b, 1024 * c + qp_fwht1024_elem(lane, tb, ta), ldxr, pack_bp)) =
                qp_fwht1024_pack(o[tb][ta]);
}

// Blocks of 1024 W, W = 2, 4, 8: one workgroup of W wavefronts per (batch row, block).
template <int W>
__global__ __launch_bounds__(64 * W < 256 ? 256 : 64 * W) void k_hadamard_chunks(const half_t *x, const int8_t *signs, int n,
                                                                                 int64_t ldx, half_t *xr, int64_t ldxr,
                                                                                 float norm, int pack_bp) {
    constexpr int block = 1024 * W;
    __shared__ __attribute__((aligned(16))) float ex[QP_FWHT_EX_FLOATS(W)];
    const int nblk = n / block;
    const int b = blockIdx.x / nblk, q = blockIdx.x - b * nblk;
    const int col0 = q * block;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (wave < W) {
        QpHad1024 H;
        H.init(lane);
        const QpHad1024In in = qp_fwht1024_fetch(x + (int64_t)b * ldx + col0 + 1024 * wave, signs + col0 + 1024 * wave, lane);
        float4_t o[2][2];
        qp_fwht1024_run(H, in, o);
        qp_fwht_park(ex, wave, lane, o);
    }
    __syncthreads();
    if (threadIdx.x < 256)
        qp_fwht_cross<W>(threadIdx.x, ex, norm * 32.0f, [&](int idx, uint2 v) {
            *reinterpret_cast<uint2 *>(xr + qp_xr_index(b, col0 + idx, ldxr, pack_bp)) = v;
        });
}

static inline bool qp_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

qp_status qp_launch_hadamard(const void *x, const int8_t *signs, int B, int n, int block, int64_t ldx,
                             void *xr, int64_t ldxr, int pack_bp, hipStream_t st) {
    const float norm = 1.0f / sqrtf((float)block);
    const int grid = B * (n / block);
    // the register kernel loads 8/16-byte pieces
    const bool vec_ok = qp_aligned16(x) && qp_aligned16(signs) && ldx % 8 == 0;
#define QP_HAD(V, W)                                                                                     \
    hipLaunchKernelGGL((k_hadamard_reg<V, W>), dim3(grid), dim3(64 * W), 0, st, (const half_t *)x, signs, n, \
                       ldx, (half_t *)xr, ldxr, norm, pack_bp)
    if (vec_ok && block == 1024 && (reinterpret_cast<uintptr_t>(xr) & 7) == 0 && ldxr % 4 == 0) {
        const int items = grid;
        hipLaunchKernelGGL(k_hadamard_1024, dim3((items + 3) / 4), dim3(256), 0, st, (const half_t *)x, signs, n, ldx,
                           (half_t *)xr, ldxr, pack_bp, items);
        return qp_check_launch();
    }
    if (vec_ok && (block == 2048 || block == 4096 || block == 8192) && (reinterpret_cast<uintptr_t>(xr) & 7) == 0 &&
        ldxr % 4 == 0) {
#define QP_HADC(W)                                                                                              \
    hipLaunchKernelGGL((k_hadamard_chunks<W>), dim3(grid), dim3(64 * W < 256 ? 256 : 64 * W), 0, st, (const half_t *)x, \
                       signs, n, ldx, (half_t *)xr, ldxr, norm, pack_bp)
        if (block == 2048) QP_HADC(2);
        else if (block == 4096) QP_HADC(4);
        else QP_HADC(8);
#undef QP_HADC
        return qp_check_launch();
    }
    if (vec_ok && block >= 256 && block <= 16384) {
        switch (block) {
            case 256: QP_HAD(4, 1); break;
            case 512: QP_HAD(4, 2); break;
            case 1024: QP_HAD(4, 4); break;
            case 2048: QP_HAD(8, 4); break;
            case 4096: QP_HAD(8, 8); break;
            case 8192: QP_HAD(16, 8); break;
            default: QP_HAD(16, 16); break;
        }
        return qp_check_launch();
    }
#undef QP_HAD
    int threads = block / 2;
    if (threads < 64) threads = 64;
    if (threads > 1024) threads = 1024;
    hipLaunchKernelGGL(k_hadamard_lds, dim3(grid), dim3(threads), (size_t)block * sizeof(float), st,
                       (const half_t *)x, signs, n, block, ldx, (half_t *)xr, ldxr, norm, pack_bp);
    return qp_check_launch();
}

// Activations that are already rotated, copied from [B, ldx] into the fragment order of the
// matrix-core kernel (the inverse of qp_xr_index): one thread per 16-byte piece of the
// destination, so that every wavefront writes one whole fragment (a contiguous KiB) and reads
// 64 pieces of 16 bytes whose cache lines its neighbours read next (x is small and stays in L2;
// the other way round - coalesced reads, scattered 16-byte writes - took twice as long).
// The batch columns B .. pack_bp - 1 are written as zeros.
__global__ __launch_bounds__(256) void k_pack_x(const half_t *x, int B, int ncols, int64_t ldx, half_t *xp, int lt) {
    // destination piece d = (C * NXF + n) * 64 + 16 g + (b << lt) + t, TT = 1 << lt steps per fragment
    const int d = blockIdx.x * blockDim.x + threadIdx.x;
    const int nxf_log = 5 - lt;
    const int nbc = (ncols + 1023) >> 10;   // a last block of fewer than 1024 columns is filled up with zeros
    if (d >= (nbc << (nxf_log + 6))) return;
    const int lane = d & 63, frag = d >> 6;
    const int n = frag & ((1 << nxf_log) - 1), C = frag >> nxf_log;
    const int g = lane >> 4, j = lane & 15;
    const int b = j >> lt, t = j & ((1 << lt) - 1);
    u32x4_t v = u32x4_t{0u, 0u, 0u, 0u};
    const int col = 1024 * C + 256 * g + 8 * ((n << lt) + t);
    if (b < B && col < ncols) v = *reinterpret_cast<const u32x4_t *>(x + (int64_t)b * ldx + col);
    reinterpret_cast<u32x4_t *>(xp)[d] = v;
}

qp_status qp_launch_pack_x(const void *x, int B, int n, int64_t ldx, void *xp, int pack_bp, hipStream_t st) {
    const int lt = 4 - __builtin_ctz(pack_bp);   // log2 of the steps per fragment, 16 / pack_bp
    const int nbc = (n + 1023) / 1024;
    const int total = nbc << (5 - lt + 6);
    hipLaunchKernelGGL(k_pack_x, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const half_t *)x, B, n, ldx,
                       (half_t *)xp, lt);
    return qp_check_launch();
}
