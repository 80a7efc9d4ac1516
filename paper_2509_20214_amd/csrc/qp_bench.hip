// Measurement aids (no part of the method): the two yardsticks the benchmark reports beside every
// quantized layer - what a kernel that only streams the same number of bytes takes on this chip, and
// what an empty launch takes.  A layer's packed codes are read once, so no kernel that computes the
// layer can be faster than the first; the second is the floor under any kernel at all.
#include "qp_internal.h"

// One wavefront reads P contiguous KiB per round with P 128-bit loads issued back to back (the
// access pattern of the fused kernel: one native block is P KiB), rounds dealt to the wavefronts of
// the grid; non-temporal like the weight stream.  The sink (4 bytes of scratch) keeps the loads alive:
// it is written only if the XOR of everything a thread read happens to equal one constant.
template <int P>
__global__ __launch_bounds__(1024) void k_stream_read(const u32x4_t *p, int64_t chunks, int64_t tail16, uint32_t *sink) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    uint32_t acc = 0;
    for (int64_t c = wave; c < chunks; c += nwaves) {
        const u32x4_t *src = p + c * (P * 64) + lane;
        u32x4_t q[P];
#pragma unroll
        for (int k = 0; k < P; ++k) q[k] = __builtin_nontemporal_load(src + k * 64);
#pragma unroll
        for (int k = 0; k < P; ++k) acc ^= q[k][0] ^ q[k][1] ^ q[k][2] ^ q[k][3];
    }
    // what is left after the whole chunks (fewer than P * 64 pieces): the first wavefronts, one piece per lane
    if (wave * 64 + lane < tail16) {
        const u32x4_t v = __builtin_nontemporal_load(p + chunks * (P * 64) + wave * 64 + lane);
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;   // (data-dependent, so the loads cannot be dropped; sink is scratch)
}

extern "C" qp_status qp_bench_stream_read(const void *data, size_t bytes, void *sink, void *hip_stream) {
    if (!data || !sink) return QP_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0) return QP_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(data) & 15) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0) return QP_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t n16 = (int64_t)(bytes / 16);
    // pieces per wavefront and round: enough that one round of 256 x 16 wavefronts covers the buffer, at most 8
    const int64_t kib = (n16 + 63) / 64;
    int P = (int)((kib + 4095) / 4096);
    if (P < 1) P = 1;
    if (P > 8) P = 8;
    const int64_t chunks = n16 / (P * 64), tail16 = n16 - chunks * (P * 64);
    // wavefronts: one per chunk up to 16 per workgroup on 256 workgroups (one workgroup per compute unit)
    int64_t per_wg = (chunks + 255) / 256;
    if (per_wg < 1) per_wg = 1;
    if (per_wg > 16) per_wg = 16;
    const dim3 grid(256), block((unsigned)(64 * per_wg));
#define QP_STREAM(PP) \
    hipLaunchKernelGGL((k_stream_read<PP>), grid, block, 0, st, (const u32x4_t *)data, chunks, tail16, (uint32_t *)sink)
    switch (P) {
        case 1: QP_STREAM(1); break;
        case 2: QP_STREAM(2); break;
        case 3: QP_STREAM(3); break;
        case 4: QP_STREAM(4); break;
        case 5: QP_STREAM(5); break;
        case 6: QP_STREAM(6); break;
        case 7: QP_STREAM(7); break;
        default: QP_STREAM(8); break;
    }
#undef QP_STREAM
    return qp_check_launch();
}

__global__ void k_empty() {}

extern "C" qp_status qp_bench_empty_launch(void *hip_stream) {
    hipLaunchKernelGGL(k_empty, dim3(256), dim3(1024), 0, static_cast<hipStream_t>(hip_stream));
    return qp_check_launch();
}
