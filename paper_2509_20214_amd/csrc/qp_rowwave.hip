// Layout-agnostic kernels: dequantize-only, and the fused layer with one wavefront
// per output row (vector ALU dot products, wavefront-shuffle reduction).  They read
// codes through qp_dword_ptr, so they serve the canonical row-major layout as well
// as the native one, for any N that is a multiple of 8 (256 for the trellis).
#include "qp_internal.h"

// ---------------------------------------------------------------- dequantize only
// One thread decodes 8 consecutive weights of one row and writes them as one
// 16-byte store (Appendix D, dequantization-only kernels).
template <int S, int CB>
__global__ __launch_bounds__(1024) void k_dequant(QpW w, uint16_t *out) {
    using T = QpTraits<S, CB>;
    __shared__ __attribute__((aligned(16))) uint16_t lut[T::LUT_HALVES];
    qp_stage_lut<T::LUT_HALVES>(w.lut, lut);
    __syncthreads();
    const int groups_per_row = w.N >> 3;
    const int64_t total = (int64_t)w.M * groups_per_row;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        int row = (int)(t / groups_per_row);
        int grp = (int)(t - (int64_t)row * groups_per_row);
        uint16_t v[8];
        qp_group_decode<S, CB>(w, row, grp, lut, v);
        u32x4_t o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<u32x4_t *>(out + (int64_t)row * w.N + (int64_t)grp * 8) = o;
    }
}

qp_status qp_launch_dequant(const QpW &w, int scheme, int cb, void *out, hipStream_t st) {
    int64_t total = (int64_t)w.M * (w.N / 8);
    int blocks = (int)((total + 1023) / 1024);
    if (blocks > 256 * 2) blocks = 256 * 2;
#define CALL(S, C) hipLaunchKernelGGL((k_dequant<S, C>), dim3(blocks), dim3(1024), 0, st, w, (uint16_t *)out)
    QP_DISPATCH_SCHEME(scheme, cb, CALL);
#undef CALL
    return qp_check_launch();
}

// ------------------------------------------------------------------ fused layer
// y[b, j] = s[j] * sum_i x[b, i] W^[j, i]  (Section 3.3).  A workgroup of 16
// wavefronts stages the table once, then each wavefront walks whole rows: lane l
// decodes weight groups l, l+64, ... and multiplies them with the matching 16 bytes
// of every activation row; partial sums meet in a butterfly of wavefront shuffles.
template <int S, int CB, int BT>
__global__ __launch_bounds__(1024) void k_linear_rowwave(QpW w, const half_t *x, int B, int64_t ldx,
                                                         half_t *y, int64_t ldy) {
    using T = QpTraits<S, CB>;
    __shared__ __attribute__((aligned(16))) uint16_t lut[T::LUT_HALVES];
    qp_stage_lut<T::LUT_HALVES>(w.lut, lut);
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int groups_per_row = w.N >> 3;
    for (int row = blockIdx.x * 16 + wave; row < w.M; row += gridDim.x * 16) {
        float acc[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) acc[b] = 0.f;
        for (int grp = lane; grp < groups_per_row; grp += 64) {
            uint16_t v[8];
            qp_group_decode<S, CB>(w, row, grp, lut, v);
            float wf[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) wf[e] = qp_half_bits_to_float(v[e]);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                if (b < B) {
                    half8_t xv = *reinterpret_cast<const half8_t *>(x + (int64_t)b * ldx + (int64_t)grp * 8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[b] = __builtin_fmaf(wf[e], (float)xv[e], acc[b]);
                }
            }
        }
        float s = qp_half_bits_to_float(w.scales[row]);
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float a = acc[b];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) a += __shfl_xor(a, m, 64);
            if (lane == 0 && b < B) y[(int64_t)b * ldy + row] = (half_t)(s * a);
        }
    }
}

qp_status qp_launch_linear_rowwave(const QpW &w, int scheme, int cb, const void *x, int B, int64_t ldx,
                                   void *y, int64_t ldy, hipStream_t st) {
    int blocks = (w.M + 15) / 16;
    if (blocks > 256) blocks = 256;
#define CALL_BT(S, C, BT)                                                                      \
    hipLaunchKernelGGL((k_linear_rowwave<S, C, BT>), dim3(blocks), dim3(1024), 0, st, w,        \
                       (const half_t *)x, B, ldx, (half_t *)y, ldy)
#define CALL(S, C)                                   \
    do {                                             \
        if (B <= 1) CALL_BT(S, C, 1);                \
        else if (B <= 2) CALL_BT(S, C, 2);           \
        else if (B <= 4) CALL_BT(S, C, 4);           \
        else if (B <= 8) CALL_BT(S, C, 8);           \
        else CALL_BT(S, C, 16);                      \
    } while (0)
    QP_DISPATCH_SCHEME(scheme, cb, CALL);
#undef CALL
#undef CALL_BT
    return qp_check_launch();
}
