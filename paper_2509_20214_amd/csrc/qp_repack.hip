// One-time canonical -> native reshuffle of the code bytes (16-byte pieces).
#include "qp_internal.h"

// Thread t moves native piece t: block = t / (64*P), piece p, lane l = 16 g + i.
__global__ void k_repack(QpW src, int span_bytes, u32x4_t *dst) {
    const int P = span_bytes / 16;
    const int64_t total = (int64_t)(src.M / 16) * src.nbc * 64 * P;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        int64_t blk = t / (64 * P);
        int rem = (int)(t - blk * 64 * P);
        int p = rem >> 6, l = rem & 63;
        int g = l >> 4, i = l & 15;
        int R = (int)(blk / src.nbc), C = (int)(blk - (int64_t)R * src.nbc);
        int row = R * 16 + i;
        int64_t byte_off = (int64_t)(C * 4 + g) * span_bytes + p * 16;
        dst[t] = *reinterpret_cast<const u32x4_t *>(src.codes + (int64_t)row * src.row_stride + byte_off);
    }
}

qp_status qp_launch_repack(const QpW &src, int span_bytes, void *dst, hipStream_t st) {
    int64_t total = (int64_t)(src.M / 16) * src.nbc * 64 * (span_bytes / 16);
    int blocks = (int)((total + 255) / 256);
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(k_repack, dim3(blocks), dim3(256), 0, st, src, span_bytes, (u32x4_t *)dst);
    return qp_check_launch();
}
