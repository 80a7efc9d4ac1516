// Code book construction by Lloyd's algorithm (Appendix C.1 / C.2 / C.3.1, "Codebook
// construction": 1-D k-means for the scalar tables, 2-D k-means for the vector tables and for
// the small table of the trellis quantizer's hybrid code book).
//
// One iteration = two launches on the caller's stream, all iterations enqueued up front:
//   k_kmeans_assign  every thread takes SPT samples at a time, finds their nearest centres
//                    (fp32; d = fma(dy, dy, dx * dx); ties: the lowest index) from the LDS copy
//                    of the centres and adds the samples into the workgroup's LDS accumulators
//                    (sum per coordinate, count); the workgroup then writes its partial sums.
//   k_kmeans_update  one workgroup adds the partial sums per centre in a fixed order in fp64,
//                    divides, measures the total squared movement, and raises `done` when it is
//                    <= tol; later launches of both kernels return at once when `done` is set,
//                    so no host synchronisation is needed between iterations.
// A cluster without samples keeps its centre.
#include "qp_internal.h"

#define QP_KM_THREADS 256
#define QP_KM_MAX_GRID 512
#define QP_KM_SPT 4   // samples per thread and trip through the centres

struct QpKmHeader {     // first 64 bytes of the workspace
    int32_t done;
    int32_t iters;
    double inertia;     // of the last assignment
    double moved;       // of the last update
    int32_t pad[10];
};

template <int D>
__global__ __launch_bounds__(QP_KM_THREADS) void k_kmeans_assign(const float *x, int64_t n, const float *centres, int k,
                                                                 QpKmHeader *hdr, float *psum, uint32_t *pcount,
                                                                 double *pinertia, int32_t *assign_out) {
    if (hdr->done) return;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    float *c = reinterpret_cast<float *>(lds);            // [k][D]
    float *sum = c + k * D;                               // [k][D]
    uint32_t *cnt = reinterpret_cast<uint32_t *>(sum + k * D);   // [k]
    __shared__ double red[QP_KM_THREADS / 64];
    for (int i = threadIdx.x; i < k * D; i += blockDim.x) {
        c[i] = centres[i];
        sum[i] = 0.f;
    }
    for (int i = threadIdx.x; i < k; i += blockDim.x) cnt[i] = 0u;
    __syncthreads();
    double inertia = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < n; i0 += stride * QP_KM_SPT) {
        float px[QP_KM_SPT], py[QP_KM_SPT], best[QP_KM_SPT];
        int bc[QP_KM_SPT];
#pragma unroll
        for (int s = 0; s < QP_KM_SPT; ++s) {
            const int64_t i = i0 + s * stride;
            const bool live = i < n;
            if (D == 2) {
                const float2 v = live ? reinterpret_cast<const float2 *>(x)[i] : make_float2(0.f, 0.f);
                px[s] = v.x;
                py[s] = v.y;
            } else {
                px[s] = live ? x[i] : 0.f;
                py[s] = 0.f;
            }
            best[s] = 3.4e38f;
            bc[s] = 0;
        }
        for (int cc = 0; cc < k; ++cc) {
            const float cx = c[cc * D], cy = (D == 2) ? c[cc * D + 1] : 0.f;
#pragma unroll
            for (int s = 0; s < QP_KM_SPT; ++s) {
                const float dx = px[s] - cx, dy = py[s] - cy;
                const float dist = (D == 2) ? __builtin_fmaf(dy, dy, dx * dx) : dx * dx;
                if (dist < best[s]) {
                    best[s] = dist;
                    bc[s] = cc;
                }
            }
        }
#pragma unroll
        for (int s = 0; s < QP_KM_SPT; ++s) {
            const int64_t i = i0 + s * stride;
            if (i < n) {
                atomicAdd(&sum[bc[s] * D], px[s]);
                if (D == 2) atomicAdd(&sum[bc[s] * D + 1], py[s]);
                atomicAdd(&cnt[bc[s]], 1u);
                inertia += (double)best[s];
                if (assign_out) assign_out[i] = bc[s];
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < k * D; i += blockDim.x) psum[(int64_t)blockIdx.x * k * D + i] = sum[i];
    for (int i = threadIdx.x; i < k; i += blockDim.x) pcount[(int64_t)blockIdx.x * k + i] = cnt[i];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) inertia += __shfl_xor(inertia, m, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = inertia;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < QP_KM_THREADS / 64; ++w) t += red[w];
        pinertia[blockIdx.x] = t;
    }
}

template <int D>
__global__ __launch_bounds__(1024) void k_kmeans_update(float *centres, int k, int grid, float tol, QpKmHeader *hdr,
                                                        const float *psum, const uint32_t *pcount,
                                                        const double *pinertia, uint16_t *centres_f16,
                                                        double *stats_out) {
    if (hdr->done) return;
    __shared__ double red[16];
    double moved = 0.0;
    for (int cc = threadIdx.x; cc < k; cc += blockDim.x) {
        uint64_t count = 0;
        double s0 = 0.0, s1 = 0.0;
        for (int g = 0; g < grid; ++g) {   // fixed order
            count += pcount[(int64_t)g * k + cc];
            s0 += (double)psum[((int64_t)g * k + cc) * D];
            if (D == 2) s1 += (double)psum[((int64_t)g * k + cc) * D + 1];
        }
        if (count > 0) {
            const float n0 = (float)(s0 / (double)count), o0 = centres[cc * D];
            moved += ((double)n0 - (double)o0) * ((double)n0 - (double)o0);
            centres[cc * D] = n0;
            if (D == 2) {
                const float n1 = (float)(s1 / (double)count), o1 = centres[cc * D + 1];
                moved += ((double)n1 - (double)o1) * ((double)n1 - (double)o1);
                centres[cc * D + 1] = n1;
            }
        }
        if (centres_f16) {
            centres_f16[cc * D] = __builtin_bit_cast(uint16_t, (half_t)centres[cc * D]);
            if (D == 2) centres_f16[cc * D + 1] = __builtin_bit_cast(uint16_t, (half_t)centres[cc * D + 1]);
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) moved += __shfl_xor(moved, m, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = moved;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0, inertia = 0.0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += red[w];
        for (int g = 0; g < grid; ++g) inertia += pinertia[g];
        hdr->iters += 1;
        hdr->inertia = inertia;
        hdr->moved = t;
        if (t <= (double)tol) hdr->done = 1;
        if (stats_out) {
            stats_out[0] = inertia;
            stats_out[1] = (double)hdr->iters;
            stats_out[2] = t;
        }
    }
}

__global__ void k_kmeans_reset(QpKmHeader *hdr) {
    if (threadIdx.x == 0) {
        hdr->done = 0;
        hdr->iters = 0;
        hdr->inertia = 0.0;
        hdr->moved = 0.0;
    }
}

static int qp_kmeans_grid(int64_t n) {
    int64_t g = (n + (int64_t)QP_KM_THREADS * QP_KM_SPT - 1) / ((int64_t)QP_KM_THREADS * QP_KM_SPT);
    if (g < 1) g = 1;
    if (g > QP_KM_MAX_GRID) g = QP_KM_MAX_GRID;
    return (int)g;
}

size_t qp_kmeans_workspace(int k, int d) {
    return sizeof(QpKmHeader) + (size_t)QP_KM_MAX_GRID * k * d * sizeof(float) + (size_t)QP_KM_MAX_GRID * k * sizeof(uint32_t) +
           (size_t)QP_KM_MAX_GRID * sizeof(double);
}

qp_status qp_launch_kmeans(const float *x, int64_t n, int d, float *centres, int k, int max_iter, float tol,
                           void *workspace, int32_t *assign_out, uint16_t *centres_f16, double *stats_out,
                           hipStream_t st) {
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    QpKmHeader *hdr = reinterpret_cast<QpKmHeader *>(ws);
    double *pinertia = reinterpret_cast<double *>(ws + sizeof(QpKmHeader));
    float *psum = reinterpret_cast<float *>(ws + sizeof(QpKmHeader) + (size_t)QP_KM_MAX_GRID * sizeof(double));
    uint32_t *pcount = reinterpret_cast<uint32_t *>(psum + (size_t)QP_KM_MAX_GRID * k * d);
    const int grid = qp_kmeans_grid(n);
    const size_t lds = (size_t)k * d * 2 * sizeof(float) + (size_t)k * sizeof(uint32_t);
    if (lds > 65536) {   // k = 4096 pairs: 80 KiB of the 160 KiB
        static bool raised = false;
        if (!raised) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_kmeans_assign<1>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 98304);
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_kmeans_assign<2>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 98304);
            raised = true;
        }
    }
    hipLaunchKernelGGL(k_kmeans_reset, dim3(1), dim3(64), 0, st, hdr);
    const int upd_threads = k >= 1024 ? 1024 : ((k + 63) / 64) * 64;
    for (int it = 0; it < max_iter; ++it) {
        if (d == 1) {
            hipLaunchKernelGGL((k_kmeans_assign<1>), dim3(grid), dim3(QP_KM_THREADS), lds, st, x, n, centres, k, hdr, psum,
                               pcount, pinertia, assign_out);
            hipLaunchKernelGGL((k_kmeans_update<1>), dim3(1), dim3(upd_threads), 0, st, centres, k, grid, tol, hdr, psum,
                               pcount, pinertia, centres_f16, stats_out);
        } else {
            hipLaunchKernelGGL((k_kmeans_assign<2>), dim3(grid), dim3(QP_KM_THREADS), lds, st, x, n, centres, k, hdr, psum,
                               pcount, pinertia, assign_out);
            hipLaunchKernelGGL((k_kmeans_update<2>), dim3(1), dim3(upd_threads), 0, st, centres, k, grid, tol, hdr, psum,
                               pcount, pinertia, centres_f16, stats_out);
        }
    }
    return qp_check_launch();
}
