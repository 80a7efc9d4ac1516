// Fused dequantize-and-multiply on the native layout (Section 3.3 "Kernel
// implementation": weights traversed once, decoded in registers, activations reused).
//
// Work unit: one native block = 16 rows x 1024 columns, owned by one wavefront.
// Lane l = 16 g + i holds row i, columns 256 g .. 256 g + 255 as P 16-byte pieces,
// fetched with P fully coalesced 128-bit loads issued before any decode.  The lane
// decodes its 256 weights in 32 steps of 8; step s of all 64 lanes is one A operand
// (16 rows x 32 k) of v_mfma_f32_16x16x32_f16, k = (g, e) <-> column 256 g + 8 s + e.
//
// The B operand (32 k x 16 columns) carries the activations.  With a batch of B <= 16
// only B of its 16 columns are needed, so the spare columns carry the activations of
// *other steps*: column j holds batch row j / TT and the x chunk of step s0 + j % TT.
// One coalesced 16-byte load per lane then serves TT consecutive steps; step s0 + t
// accumulates into its own accumulator acc[t], of which only the columns with
// j % TT == t are meaningful.  Summing those columns over t at the end gives the dot
// products.  TT = min(16 / Bp, 8) with Bp = B rounded up to a power of two.
//
// A workgroup owns a contiguous range of 16-row blocks and walks it in passes of G
// row blocks; the G * (N / 1024) units of a pass are dealt round-robin to the
// wavefronts, each unit's column-selected partial sums go to LDS, and after a barrier
// the workgroup adds them up, applies the per-row scale and stores fp16.
#include "qp_internal.h"

#define QP_UMAX 32  // units per pass (LDS: 1 KiB each)

#ifdef QP_TRACE  // development builds only: per-wavefront timestamps of the kernel's phases
__device__ uint64_t *qp_trace_buf;
extern "C" void qp_debug_set_trace(void *p) { (void)hipMemcpyToSymbol(HIP_SYMBOL(qp_trace_buf), &p, sizeof(p)); }
#define QP_T(slot)                                                                                   \
    do {                                                                                             \
        if ((threadIdx.x & 63) == 0)                                                                 \
            qp_trace_buf[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + (slot)] = __builtin_amdgcn_s_memtime(); \
    } while (0)
#define QP_TID()                                                                                     \
    do {                                                                                             \
        if ((threadIdx.x & 63) == 0)                                                                 \
            qp_trace_buf[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + 7] =                   \
                ((uint64_t)__builtin_amdgcn_s_getreg(63492) << 32) | __builtin_amdgcn_s_getreg(63508); \
    } while (0)
#else
#define QP_T(slot)
#define QP_TID()
#endif

// Compile-time bit-field extraction from the lane's P 16-byte pieces, seen as one
// little-endian stream of 128 P bits.  Every index is a constant once the step loop is
// unrolled, so the pieces stay in registers.  WRAP: the stream is circular (tail-biting
// trellis tile); otherwise the caller guarantees that the field lies inside it.
template <int P>
__device__ __forceinline__ uint32_t qp_dw(const u32x4_t (&q)[P], int idx) {
    return q[idx >> 2][idx & 3];
}

template <int P, bool WRAP>
__device__ __forceinline__ uint32_t qp_field(const u32x4_t (&q)[P], int bitpos, int nbits) {
    const int i0 = bitpos >> 5, r = bitpos & 31;
    const uint32_t mask = (nbits == 32) ? 0xffffffffu : ((1u << nbits) - 1u);
    if (r + nbits <= 32) return (qp_dw<P>(q, i0) >> r) & mask;
    const int i1 = WRAP ? ((i0 + 1) % (4 * P)) : (i0 + 1);
    return __builtin_amdgcn_alignbit(qp_dw<P>(q, i1), qp_dw<P>(q, i0), r) & mask;
}

// Decode the 8 weights of step s (columns 8 s .. 8 s + 7 of the lane's 256) into an
// MFMA operand.
template <int S, int CB, int P>
__device__ __forceinline__ half8_t qp_decode_step(const u32x4_t (&q)[P], int s, const uint16_t *lut) {
    half8_t a;
    if (S == QP_SQ) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            a[e] = __builtin_bit_cast(half_t, lut[qp_field<P, false>(q, (8 * s + e) * CB, CB)]);
    } else if (S == QP_VQ) {
        const uint32_t *lut2 = reinterpret_cast<const uint32_t *>(lut);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t p = lut2[qp_field<P, false>(q, (4 * s + c) * CB, CB)];
            half2_t h = __builtin_bit_cast(half2_t, p);
            a[2 * c] = h[0];
            a[2 * c + 1] = h[1];
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            a[e] = __builtin_bit_cast(half_t, lut[qp_field<P, true>(q, (8 * s + e) * CB, 16)]);
    }
    return a;
}

template <int S, int CB, int BP>
__global__ __launch_bounds__(1024) void k_linear_mfma(QpW w, const half_t *x, int B, int64_t ldx, half_t *y,
                                                      int64_t ldy, int G) {
    using T = QpTraits<S, CB>;
    constexpr int P = T::PIECES;
    constexpr int TT = (16 / BP < 8) ? 16 / BP : 8;  // steps per activation fragment
    __shared__ __attribute__((aligned(16))) uint16_t lut[T::LUT_HALVES];
    __shared__ __attribute__((aligned(16))) float red[QP_UMAX][64][4];
    QP_T(0);
    QP_TID();
    qp_stage_lut<T::LUT_HALVES>(w.lut, lut);
    __syncthreads();
    QP_T(1);

    const int nw = blockDim.x >> 6;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane >> 4, j = lane & 15;
    const int tj = j % TT;
    int bj = j / TT;
    if (bj >= B) bj = B - 1;  // spare columns re-read a valid row; their results are never used
    const int nbc = w.nbc;
    const int rbk = w.M >> 4;
    // balanced contiguous partition of the row blocks over the workgroups
    const int rb_begin = (int)((int64_t)rbk * blockIdx.x / gridDim.x);
    const int rb_end = (int)((int64_t)rbk * (blockIdx.x + 1) / gridDim.x);
    const half_t *xlane = x + (int64_t)bj * ldx + 256 * g + 8 * tj;

    for (int rb0 = rb_begin; rb0 < rb_end; rb0 += G) {
        const int gcount = (rb_end - rb0 < G) ? (rb_end - rb0) : G;
        const int units = gcount * nbc;
        for (int u = wave; u < units; u += nw) {
            const int slot = u / nbc, C = u - slot * nbc;
            const u32x4_t *blk = reinterpret_cast<const u32x4_t *>(
                w.codes + ((int64_t)(rb0 + slot) * nbc + C) * T::BLOCK_BYTES);
            u32x4_t q[P];
#pragma unroll
            for (int p = 0; p < P; ++p) q[p] = __builtin_nontemporal_load(blk + p * 64 + lane);
            const half_t *xu = xlane + (int64_t)C * 1024;
            half8_t xf = *reinterpret_cast<const half8_t *>(xu);
            float4_t acc[TT];
#pragma unroll
            for (int t = 0; t < TT; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
#ifdef QP_TRACE
            if (u == wave && rb0 == rb_begin) {
                if (q[0][0] == 0x12345 && q[P - 1][3] == 0x777) acc[0][0] = 1.f;  // forces the loads to have landed
                QP_T(2);
            }
#endif
#pragma unroll
            for (int s = 0; s < 32; ++s) {
                if (s > 0 && s % TT == 0) xf = *reinterpret_cast<const half8_t *>(xu + 8 * s);
                half8_t a = qp_decode_step<S, CB, P>(q, s, lut);
                acc[s % TT] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, xf, acc[s % TT], 0, 0, 0);
            }
            float4_t v = acc[0];
#pragma unroll
            for (int t = 1; t < TT; ++t)
                if (tj == t) v = acc[t];
            *reinterpret_cast<float4_t *>(&red[u][lane][0]) = v;
            QP_T(3);
        }
        QP_T(4);
        __syncthreads();
        QP_T(5);
        // outputs of this pass: (slot, b, i); consecutive threads take consecutive rows
        for (int o = threadIdx.x; o < gcount * 16 * B; o += blockDim.x) {
            const int i = o & 15;
            const int b = (o >> 4) % B;
            const int slot = (o >> 4) / B;
            float sum = 0.f;
            for (int C = 0; C < nbc; ++C) {
                const float *r = &red[slot * nbc + C][16 * (i >> 2) + b * TT][i & 3];
#pragma unroll
                for (int t = 0; t < TT; ++t) sum += r[4 * t];
            }
            const int row = (rb0 + slot) * 16 + i;
            y[(int64_t)b * ldy + row] = (half_t)(qp_half_bits_to_float(w.scales[row]) * sum);
        }
        __syncthreads();
    }
    QP_T(6);
}

qp_status qp_launch_linear_mfma(const QpW &w, int scheme, int cb, const void *x, int B, int64_t ldx, void *y,
                                int64_t ldy, hipStream_t st) {
    const int nbc = w.nbc, rbk = w.M / 16;
    if (nbc < 1 || nbc > QP_UMAX) return QP_ERR_UNSUPPORTED;
    int grid = rbk < 256 ? rbk : 256;
    int rb_per_wg = (rbk + grid - 1) / grid;
    int G = QP_UMAX / nbc;
    if (G > rb_per_wg) G = rb_per_wg;
    int units = G * nbc;
    int nw = units < 16 ? units : 16;
    if (scheme == QP_TCQ && nw < 16) nw = 16;  // all 1024 threads help staging the 128 KiB table
    if (nw < 4) nw = 4;
#define CALL_BP(S, C, BP)                                                                              \
    hipLaunchKernelGGL((k_linear_mfma<S, C, BP>), dim3(grid), dim3(64 * nw), 0, st, w, (const half_t *)x, B, \
                       ldx, (half_t *)y, ldy, G)
#define CALL(S, C)                                   \
    do {                                             \
        if (B <= 1) CALL_BP(S, C, 1);                \
        else if (B <= 2) CALL_BP(S, C, 2);           \
        else if (B <= 4) CALL_BP(S, C, 4);           \
        else if (B <= 8) CALL_BP(S, C, 8);           \
        else CALL_BP(S, C, 16);                      \
    } while (0)
    QP_DISPATCH_SCHEME(scheme, cb, CALL);
#undef CALL
#undef CALL_BP
    return qp_check_launch();
}
