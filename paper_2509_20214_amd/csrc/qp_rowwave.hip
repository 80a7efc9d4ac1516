// Layout-agnostic kernels: dequantize-only, and the fused layer with one wavefront
// per output row (vector ALU dot products, wavefront-shuffle reduction).  They read
// codes through qp_dword_ptr, so they serve the canonical row-major layout as well
// as the native one, for any N that is a multiple of 8 (256 for the trellis).
#include "qp_internal.h"
#include "qp_fwht.h"

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
// In-kernel rotation: the longest row it takes, and whether a scheme's table leaves LDS room for the
// parked chunks of a block of more than 1024.
#define QP_ROWWAVE_ROT_MAX_N 8192
template <int S, int CB>
constexpr bool qp_rowwave_parks() { return QpTraits<S, CB>::LUT_HALVES * 2 <= 65536; }

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

// The same at batch 1 with the rotation of Section 3.3 inside: tiny layers, where a second launch
// costs as much as the layer itself.  N / 1024 <= 8 wavefronts transform a chunk of 1024 each on the
// matrix cores (the code of the stand-alone kernels, hence the same bits) while the table is staged;
// the rotated row stays in LDS and every wavefront reads its rows' activations from there.
// rot_block == 1024: the chunks are the blocks.  rot_block == N: one block, finished by the butterfly
// stages across the chunks (only where the table leaves room to park them).
template <int S, int CB>
__global__ __launch_bounds__(1024) void k_linear_rowwave_rot(QpW w, const half_t *x, const int8_t *signs,
                                                             int rot_block, float rot_norm, half_t *y) {
    using T = QpTraits<S, CB>;
    constexpr bool CROSS = qp_rowwave_parks<S, CB>();
    __shared__ __attribute__((aligned(16))) uint16_t lut[T::LUT_HALVES];
    __shared__ __attribute__((aligned(16))) half_t xs[QP_ROWWAVE_ROT_MAX_N];
    __shared__ __attribute__((aligned(16))) uint32_t had[1024];
    __shared__ __attribute__((aligned(16))) float ex[CROSS ? QP_FWHT_EX_FLOATS(QP_ROWWAVE_ROT_MAX_N / 1024) : 4];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nch = w.N >> 10;
    QpHad1024In in;
    if (wave < nch) in = qp_fwht1024_fetch(x + 1024 * wave, signs + 1024 * wave, lane);
    QpHad1024::fill(had, (int)blockDim.x);
    qp_stage_lut<T::LUT_HALVES>(w.lut, lut);
    __syncthreads();
    if (wave < nch) {
        QpHad1024 H;
        H.read(had, lane);
        float4_t o[2][2];
        qp_fwht1024_run(H, in, o);
        if (rot_block == 1024) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int ta = 0; ta < 2; ++ta)
                    *reinterpret_cast<uint2 *>(xs + 1024 * wave + qp_fwht1024_elem(lane, tb, ta)) = qp_fwht1024_pack(o[tb][ta]);
        } else if constexpr (CROSS) {
            qp_fwht_park(ex, wave, lane, o);
        }
    }
    __syncthreads();
    if constexpr (CROSS) {
        if (rot_block != 1024) {   // (uniform over the workgroup)
            if (threadIdx.x < 256) {
                auto put = [&](int idx, uint2 v) { *reinterpret_cast<uint2 *>(xs + idx) = v; };
                const float scale = rot_norm * 32.0f;
                if (nch == 2) qp_fwht_cross<2>(threadIdx.x, ex, scale, put);
                else if (nch == 4) qp_fwht_cross<4>(threadIdx.x, ex, scale, put);
                else qp_fwht_cross<8>(threadIdx.x, ex, scale, put);
            }
            __syncthreads();
        }
    }
    const int groups_per_row = w.N >> 3;
    for (int row = blockIdx.x * 16 + wave; row < w.M; row += gridDim.x * 16) {
        float acc = 0.f;
        for (int grp = lane; grp < groups_per_row; grp += 64) {
            uint16_t v[8];
            qp_group_decode<S, CB>(w, row, grp, lut, v);
            const half8_t xv = *reinterpret_cast<const half8_t *>(xs + grp * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(qp_half_bits_to_float(v[e]), (float)xv[e], acc);
        }
        const float s = qp_half_bits_to_float(w.scales[row]);
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
        if (lane == 0) y[row] = (half_t)(s * acc);
    }
}

// Whether the row kernel can rotate the activations itself: batch 1, N a multiple of 1024 up to
// QP_ROWWAVE_ROT_MAX_N, and either blocks of 1024 or one block (a power of two from 2048 on; not beside
// the 128 KiB table of the V = 1 trellis, which leaves no room to park the chunks).
bool qp_rowwave_rotates(int scheme, int cb, int N, int rot_block) {
    if (N % 1024 != 0 || N < 1024 || N > QP_ROWWAVE_ROT_MAX_N) return false;
    if (rot_block == 1024) return true;
    if (rot_block != N || (N != 2048 && N != 4096 && N != 8192)) return false;
    bool parks = false;
#define CALL(S, C) parks = qp_rowwave_parks<S, C>()
    [&]() -> qp_status { QP_DISPATCH_SCHEME(scheme, cb, CALL); return QP_OK; }();
#undef CALL
    return parks;
}

qp_status qp_launch_linear_rowwave_rot(const QpW &w, int scheme, int cb, const void *x, const int8_t *signs,
                                       int rot_block, void *y, hipStream_t st) {
    if (!qp_rowwave_rotates(scheme, cb, w.N, rot_block)) return QP_ERR_UNSUPPORTED;
    int blocks = (w.M + 15) / 16;
    if (blocks > 256) blocks = 256;
    const float rot_norm = 1.0f / sqrtf((float)rot_block);
#define CALL(S, C)                                                                                          \
    hipLaunchKernelGGL((k_linear_rowwave_rot<S, C>), dim3(blocks), dim3(1024), 0, st, w, (const half_t *)x, \
                       signs, rot_block, rot_norm, (half_t *)y)
    QP_DISPATCH_SCHEME(scheme, cb, CALL);
#undef CALL
    return qp_check_launch();
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
