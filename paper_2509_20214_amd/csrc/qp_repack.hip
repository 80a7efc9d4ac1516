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
        // spans of the last column block beyond N (N % 1024 != 0) are padding: zero bytes
        u32x4_t v = u32x4_t{0u, 0u, 0u, 0u};
        if ((C * 4 + g) * 256 < src.N) v = *reinterpret_cast<const u32x4_t *>(src.codes + (int64_t)row * src.row_stride + byte_off);
        dst[t] = v;
    }
}

qp_status qp_launch_repack(const QpW &src, int span_bytes, void *dst, hipStream_t st) {
    int64_t total = (int64_t)(src.M / 16) * src.nbc * 64 * (span_bytes / 16);
    int blocks = (int)((total + 255) / 256);
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(k_repack, dim3(blocks), dim3(256), 0, st, src, span_bytes, (u32x4_t *)dst);
    return qp_check_launch();
}

// Half-TCQ: per block row, h = nbc / 2 blocks of P = cb pieces per lane, then h blocks of
// cb + 1.  Thread t moves native piece t.
__global__ void k_repack_half(QpW src, int cb, u32x4_t *dst) {
    const int h = src.nbc >> 1;
    const int64_t lo_pieces = (int64_t)h * 64 * cb;                 // pieces of a block row's first half
    const int64_t row_pieces = lo_pieces + (int64_t)h * 64 * (cb + 1);
    const int64_t total = (int64_t)(src.M / 16) * row_pieces;
    const int64_t lo_row_bytes = (int64_t)(src.N >> 9) * (16 * cb);  // canonical bytes of a row's first half
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int R = (int)(t / row_pieces);
        int64_t rem = t - (int64_t)R * row_pieces;
        const bool hi = rem >= lo_pieces;
        if (hi) rem -= lo_pieces;
        const int P = cb + (hi ? 1 : 0);
        const int C = (int)(rem / (64 * P));          // column block inside its half
        const int r2 = (int)(rem - (int64_t)C * 64 * P);
        const int p = r2 >> 6, l = r2 & 63;
        const int g = l >> 4, i = l & 15;
        const int64_t byte_off = (hi ? lo_row_bytes : 0) + (int64_t)(C * 4 + g) * (16 * P) + p * 16;
        dst[t] = *reinterpret_cast<const u32x4_t *>(src.codes + (int64_t)(R * 16 + i) * src.row_stride + byte_off);
    }
}

qp_status qp_launch_repack_half(const QpW &src, int cb, void *dst, hipStream_t st) {
    const int64_t total = (int64_t)(src.M / 16) * (src.nbc >> 1) * 64 * (2 * cb + 1);
    int blocks = (int)((total + 255) / 256);
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(k_repack_half, dim3(blocks), dim3(256), 0, st, src, cb, (u32x4_t *)dst);
    return qp_check_launch();
}
