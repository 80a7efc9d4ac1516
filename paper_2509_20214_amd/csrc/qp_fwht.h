// Fast Walsh-Hadamard transform of one block by a group of wavefronts, shared by the
// stand-alone rotation kernel and by the fused layer kernel when it rotates its own input.
#pragma once
#include "qp_dev.h"

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


// One block of 64 V W values, transformed by W wavefronts: thread t (0 .. 64 W - 1) of the
// group loads values t V .. t V + V - 1 of src (fp16) and their signs (8/16-byte pieces: src and
// sg 16-byte aligned), and after the transform hands every scaled result to store(index in the
// block, fp16 value).  buf: 64 V W + 2 V W floats of LDS (unused when W == 1).  Threads of the
// workgroup that are not part of the group pass active = false: they only take part in the
// barrier, which every thread of the workgroup must reach.
// v * norm rounded to fp32, then to fp16: two roundings, always.  (Left to itself the compiler
// may or may not merge them into one mixed-precision instruction with a single rounding,
// depending on the surrounding code, and the two kernels that share this transform would then
// disagree in the last bit.)
__device__ __forceinline__ half_t qp_scale_round(float v, float norm) {
    float p = v * norm;
    asm volatile("" : "+v"(p));
    return (half_t)p;
}

// First half of qp_fwht_tile: the loads only (the values times their signs, fp32).
template <int V>
__device__ __forceinline__ void qp_fwht_fetch(bool active, int t, const half_t *src, const int8_t *sg, float (&v)[V]) {
#pragma unroll
    for (int k = 0; k < V; ++k) v[k] = 0.f;
    if (active) {
        if constexpr (V == 4) {
            typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
            const half4_t hv = *reinterpret_cast<const half4_t *>(src + t * V);
            const uint32_t sv = *reinterpret_cast<const uint32_t *>(sg + t * V);
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = (float)hv[k] * (float)(int8_t)(sv >> (8 * k));
        } else {
#pragma unroll
            for (int c = 0; c < V / 8; ++c) {
                const half8_t hv = reinterpret_cast<const half8_t *>(src + t * V)[c];
                const uint64_t sv = reinterpret_cast<const uint64_t *>(sg + t * V)[c];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[8 * c + k] = (float)hv[k] * (float)(int8_t)(sv >> (8 * k));
            }
        }
    }
}

// Second half: the butterflies and the stores.
template <int V, int W, class Store>
__device__ __forceinline__ void qp_fwht_finish(bool active, int t, float (&v)[V], float norm, float *buf, Store store) {
    const int lane = t & 63;
    if (active) {
        qp_fwht_regs<V>(v);
        qp_fwht_lanes<V>(v, lane);
    }
    if constexpr (W == 1) {
        if (active) {
#pragma unroll
            for (int k = 0; k < V; ++k) store(t * V + k, qp_scale_round(v[k], norm));
        }
    } else {
        if (active) {
#pragma unroll
            for (int k = 0; k < V; ++k) buf[qp_pad(t * V + k)] = v[k];
        }
        __syncthreads();
        if (active) {
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
            for (int i = 0; i < V; ++i) store((i / PER) * SPAN + t * PER + (i % PER), qp_scale_round(v[i], norm));
        }
    }
}

template <int V, int W, class Store>
__device__ __forceinline__ void qp_fwht_tile(bool active, int t, const half_t *src, const int8_t *sg, float norm,
                                             float *buf, Store store) {
    float v[V];
    qp_fwht_fetch<V>(active, t, src, sg, v);
    qp_fwht_finish<V, W>(active, t, v, norm, buf, store);
}
