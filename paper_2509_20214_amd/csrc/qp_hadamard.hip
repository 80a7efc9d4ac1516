// Online rotation of activations (Section 3.3): per block, xr = H (signs .* x) / sqrt(block),
// H the Sylvester Hadamard matrix in natural order, computed as log2(block) butterfly
// stages in fp32 and rounded once to fp16.
#include "qp_internal.h"

// Where element `col` of batch row b goes.  pack_bp == 0: row-major, b * ldxr + col.
// Otherwise the fragment order that the block kernel of the fused layer loads for a batch
// padded to pack_bp (a power of two <= 16): with TT = 16 / pack_bp steps per fragment,
// column c = 256 g + 8 s + e of column block C sits at half
// ((C * (32 / TT) + s / TT) * 64 + 16 g + b * TT + s % TT) * 8 + e,
// so that every fragment is one contiguous KiB.
__device__ __forceinline__ int64_t qp_xr_index(int b, int col, int64_t ldxr, int pack_bp) {
    if (pack_bp == 0) return (int64_t)b * ldxr + col;
    const int lt = __builtin_ctz(16 / 1) - __builtin_ctz(pack_bp);   // log2(TT) = 4 - log2(pack_bp)
    const int C = col >> 10, g = (col >> 8) & 3, s = (col >> 3) & 31, e = col & 7;
    const int n = s >> lt, t = s & ((1 << lt) - 1);
    return ((((int64_t)((C << (5 - lt)) + n) << 6) + 16 * g + (b << lt) + t) << 3) + e;
}

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
        xr[qp_xr_index(b, q * block + i, ldxr, pack_bp)] = (half_t)(buf[i] * norm);
}

// Fast path for blocks of 256..16384: thread t holds V consecutive values.  The
// butterfly stages factor over the bits of the element index e = [wave | lane | k]:
// the k bits are done in registers, the lane bits with wavefront shuffles, the wave
// bits after one transpose through LDS (each thread then holds, for V/W positions,
// the W values that differ only in the wave bits).  Stages over different bits commute.
// V and the number of wavefronts W are template parameters so that every index into the
// value array is a constant (a run-time index would push the array out of registers).
template <int V>
__device__ __forceinline__ void qp_fwht_regs(float (&v)[V]) {
#pragma unroll
    for (int h = 1; h < V; h <<= 1)
#pragma unroll
        for (int i = 0; i < V; ++i)
            if ((i & h) == 0) {
                const float a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
}

// Value of lane (l ^ (1 << M)).  Inside a row of 16 lanes the exchange is a DPP modifier
// (quad permutes for 1 and 2; a shift by 4 in each direction, each written to the banks it
// is valid for; a rotation by 8); across rows it goes through the LDS crossbar.
template <int M>
__device__ __forceinline__ float qp_lane_xor(float v) {
    const int iv = __builtin_bit_cast(int, v);
    int r;
    if constexpr (M == 0) {
        r = __builtin_amdgcn_update_dpp(0, iv, 0xB1, 0xf, 0xf, false);        // quad_perm [1,0,3,2]
    } else if constexpr (M == 1) {
        r = __builtin_amdgcn_update_dpp(0, iv, 0x4E, 0xf, 0xf, false);        // quad_perm [2,3,0,1]
    } else if constexpr (M == 2) {
        r = __builtin_amdgcn_update_dpp(iv, iv, 0x104, 0xf, 0x5, false);      // row_shl:4 into banks 0, 2
        r = __builtin_amdgcn_update_dpp(r, iv, 0x114, 0xf, 0xA, false);       // row_shr:4 into banks 1, 3
    } else if constexpr (M == 3) {
        r = __builtin_amdgcn_update_dpp(0, iv, 0x128, 0xf, 0xf, false);       // row_ror:8
    } else {
        return __shfl_xor(v, 1 << M, 64);
    }
    return __builtin_bit_cast(float, r);
}

template <int V, int M = 0>
__device__ __forceinline__ void qp_fwht_lanes(float (&v)[V], int lane) {
    if constexpr (M < 6) {
        const bool hi = (lane >> M) & 1;
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const float o = qp_lane_xor<M>(v[k]);
            v[k] = hi ? (o - v[k]) : (v[k] + o);
        }
        qp_fwht_lanes<V, M + 1>(v, lane);
    }
}

// LDS index of element e: one word of padding per 32 keeps both the stride-V writes and
// the stride-V/W reads of the transpose free of bank conflicts.
__device__ __forceinline__ int qp_pad(int e) { return e + (e >> 5); }

template <int V, int W>
__global__ __launch_bounds__(64 * W) void k_hadamard_reg(const half_t *x, const int8_t *signs, int n,
                                                         int64_t ldx, half_t *xr, int64_t ldxr, float norm,
                                                         int pack_bp) {
    constexpr int block = 64 * V * W;
    __shared__ float buf[(W > 1) ? block + block / 32 : 1];
    const int nblk = n / block;
    const int b = blockIdx.x / nblk, q = blockIdx.x - b * nblk;
    const int t = threadIdx.x, lane = t & 63;
    // V halves and V sign bytes per thread, fetched as 8- or 16-byte pieces (the launcher
    // has checked the alignment)
    float v[V];
    {
        const half_t *src = x + (int64_t)b * ldx + (int64_t)q * block + t * V;
        const int8_t *sg = signs + (int64_t)q * block + t * V;
        if constexpr (V == 4) {
            typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
            const half4_t hv = *reinterpret_cast<const half4_t *>(src);
            const uint32_t sv = *reinterpret_cast<const uint32_t *>(sg);
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = (float)hv[k] * (float)(int8_t)(sv >> (8 * k));
        } else {
#pragma unroll
            for (int c = 0; c < V / 8; ++c) {
                const half8_t hv = reinterpret_cast<const half8_t *>(src)[c];
                const uint64_t sv = reinterpret_cast<const uint64_t *>(sg)[c];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[8 * c + k] = (float)hv[k] * (float)(int8_t)(sv >> (8 * k));
            }
        }
    }
    qp_fwht_regs<V>(v);
    qp_fwht_lanes<V>(v, lane);
    const int col0 = q * block;
    if constexpr (W == 1) {
#pragma unroll
        for (int k = 0; k < V; ++k) xr[qp_xr_index(b, col0 + t * V + k, ldxr, pack_bp)] = (half_t)(v[k] * norm);
    } else {
#pragma unroll
        for (int k = 0; k < V; ++k) buf[qp_pad(t * V + k)] = v[k];
        __syncthreads();
        // element (wv, r): wv = wave bits, r in [0, 64 V); this thread takes r = t * PER + qq
        constexpr int PER = V / W;     // positions per thread
        constexpr int SPAN = 64 * V;   // elements per wave-bit value
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = buf[qp_pad((i / PER) * SPAN + t * PER + (i % PER))];
        // butterflies over wv: values that differ in wv sit PER apart in v[]
#pragma unroll
        for (int h = 1; h < W; h <<= 1)
#pragma unroll
            for (int i = 0; i < V; ++i)
                if (((i / PER) & h) == 0) {
                    const float a = v[i], c = v[i + h * PER];
                    v[i] = a + c;
                    v[i + h * PER] = a - c;
                }
#pragma unroll
        for (int i = 0; i < V; ++i)
            xr[qp_xr_index(b, col0 + (i / PER) * SPAN + t * PER + (i % PER), ldxr, pack_bp)] = (half_t)(v[i] * norm);
    }
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
