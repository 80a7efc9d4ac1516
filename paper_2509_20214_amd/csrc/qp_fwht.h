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

// The copy of the rotated activations that a layer's kernel keeps in LDS for itself (batch 1, fragment
// order) is swizzled: the 16-byte piece of lane l of a fragment sits in slot l ^ ((l >> 3) & 7).  Readers -
// one piece per lane - still cover every 128-byte row with each group of eight lanes; the writers of the
// matrix-core transform, whose sixteen lanes of a row would otherwise hit two bank pairs (eight-way conflict,
// 400 k conflict cycles per launch of 4096x14336), spread over all of them.
__device__ __forceinline__ int qp_xr_swizzle_lane(int lane) { return lane ^ ((lane >> 3) & 7); }
__device__ __forceinline__ int qp_xr_swizzled(int64_t half_index) {
    const int h = (int)half_index, slot = (h >> 3) & 63;
    return (h & ~(63 << 3)) | (qp_xr_swizzle_lane(slot) << 3);
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


// ------------------------------------------------------------------ a block of 1024 on the matrix cores
// One wavefront transforms one block of 1024 as a 32 x 32 matrix X[a][b] = x[32 a + b]:
// Y = H32 X H32 (the Sylvester matrix of order 1024 is H32 (x) H32), two passes of
// v_mfma_f32_16x16x32_f16 instead of ten butterfly stages - the six stages that cross lanes cost
// three vector operations per value each, about 350 per wavefront and block; this takes 12 matrix
// instructions and about 80 vector operations.
//   pass 1  T[a][b'] = sum_b X[a][b] H[b][b'] / 32    X: fp16 times its sign, exact; fp32 sums
//   pass 2  Y[b'][a'] = sum_a T[a][b'] H[a][a']       T = hi + lo, two fp16 numbers that carry 22 bits
//                                                      of its mantissa; hi first, then lo, fp32 sums
// The 1 / 32 = 1 / sqrt(1024) rides in pass 1's constant matrix, so T fits fp16 whenever x does.
// Pass 1's results already sit where pass 2's A operand wants them (a lane's accumulator rows become
// its k slots; the constant matrix of pass 2 is labelled to match), so nothing moves between lanes.
// Lane (g, j) = 16 g + j ends up with out[tb][ta][r] = element 32 (16 ta + j) + 16 tb + 4 g + r of the
// transformed block, r = 0 .. 3: four consecutive elements per register quadruple.
// Dword d (k slots 2 d, 2 d + 1) of lane (g, j)'s piece q of the two constant matrices: q = 0, 1 pass 1,
// column tile q; q = 2, 3 pass 2, column tile q - 2.
__device__ __forceinline__ uint32_t qp_had1024_word(int q, int lane, int d) {
    const int g = lane >> 4, c = 16 * (q & 1) + (lane & 15);
    uint32_t w = 0;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const int e = 2 * d + hh;
        const int k = (q < 2) ? 8 * g + e                                       // pass 1: k slot e of lane group g is b = 8 g + e
                              : ((e < 4) ? 4 * g + e : 16 + 4 * g + (e - 4));   // pass 2: it is a = pi(g, e)
        const uint32_t one = (q < 2) ? 0x2800u : 0x3c00u;                        // 2^-5 and 1 in fp16
        w |= (one | ((uint32_t)(__builtin_popcount(k & c) & 1) << 15)) << (16 * hh);
    }
    return w;
}

struct QpHad1024 {
    u32x4_t h1[2];   // pass 1, B operand for columns b' = 16 tb + j: H[8 g + e][b'] / 32, e = 0 .. 7
    u32x4_t h2[2];   // pass 2, B operand for columns a' = 16 ta + j: H[pi(g, e)][a'], pi(g, e) = 4 g + e, 16 + 4 g + e - 4
    // Every lane works out its own 16 dwords (about 200 vector operations: fine for a kernel that does
    // nothing else, too much for one that has a layer to compute).
    __device__ __forceinline__ void init(int lane) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                h1[t][d] = qp_had1024_word(t, lane, d);
                h2[t][d] = qp_had1024_word(2 + t, lane, d);
            }
    }
    // The workgroup works them out once, one dword per thread, into 4 KiB of LDS (1024 dwords, [q][lane][d]);
    // after a barrier every wavefront reads its copy.
    // (qp_had1024_word with q, lane and d taken from a run-time index compiles to a dozen branches on the
    // execution mask; the same dword without one: k slot 2 d of the pair, its column c, the parities of k & c and
    // (k | 1) & c - the second is the first flipped by c's lowest bit.)
    static __device__ __forceinline__ void fill(uint32_t *lds, int wgt) {   // wgt: threads of the workgroup
        for (int idx = threadIdx.x; idx < 1024; idx += wgt) {
            const uint32_t d = idx & 3, g = (idx >> 6) & 3, j = (idx >> 2) & 15, q = idx >> 8, p2 = q >> 1;
            const uint32_t k0 = (g << (3 - p2)) + 2 * d + 12 * (p2 & (d >> 1));   // pass 1: 8 g + e; pass 2: pi(g, e); e = 2 d
            const uint32_t c = 16 * (q & 1) + j;
            const uint32_t par0 = __builtin_popcount(k0 & c) & 1, par1 = par0 ^ (c & 1);
            const uint32_t one = 0x2800u + 0x1400u * p2;                          // 2^-5 (pass 1) and 1 (pass 2) in fp16
            lds[idx] = (one | (par0 << 15)) | ((one | (par1 << 15)) << 16);
        }
    }
    __device__ __forceinline__ void read(const uint32_t *lds, int lane) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            h1[t] = *reinterpret_cast<const u32x4_t *>(lds + (t * 64 + lane) * 4);
            h2[t] = *reinterpret_cast<const u32x4_t *>(lds + ((2 + t) * 64 + lane) * 4);
        }
    }
};

// The loads of one block: lane (g, i) takes x[32 (16 ta + i) + 8 g .. + 7] and the signs of the same
// elements, ta = 0, 1 (src and sg 16- and 8-byte aligned).
struct QpHad1024In {
    u32x4_t xv[2];
    uint64_t sv[2];
};
__device__ __forceinline__ QpHad1024In qp_fwht1024_fetch(const half_t *src, const int8_t *sg, int lane) {
    QpHad1024In in;
    const int g = lane >> 4, i = lane & 15;
#pragma unroll
    for (int ta = 0; ta < 2; ++ta) {
        const int off = 32 * (16 * ta + i) + 8 * g;
        in.xv[ta] = *reinterpret_cast<const u32x4_t *>(src + off);
        in.sv[ta] = *reinterpret_cast<const uint64_t *>(sg + off);
    }
    return in;
}

__device__ __forceinline__ void qp_fwht1024_run(const QpHad1024 &H, const QpHad1024In &in, float4_t (&out)[2][2]) {
    const float4_t zero = float4_t{0.f, 0.f, 0.f, 0.f};
    float4_t t1[2][2];
#pragma unroll
    for (int ta = 0; ta < 2; ++ta) {
        // sign byte 0x01 / 0xff -> bit 7; byte 2 d of the eight goes to bit 15 of dword d, byte 2 d + 1 to bit 31
        const uint32_t s_lo = (uint32_t)in.sv[ta] & 0x80808080u, s_hi = (uint32_t)(in.sv[ta] >> 32) & 0x80808080u;
        u32x4_t xa = in.xv[ta];
        xa[0] ^= __builtin_amdgcn_perm(0u, s_lo, 0x010c000cu);
        xa[1] ^= __builtin_amdgcn_perm(0u, s_lo, 0x030c020cu);
        xa[2] ^= __builtin_amdgcn_perm(0u, s_hi, 0x010c000cu);
        xa[3] ^= __builtin_amdgcn_perm(0u, s_hi, 0x030c020cu);
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
            t1[ta][tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, xa),
                                                                __builtin_bit_cast(half8_t, H.h1[tb]), zero, 0, 0, 0);
    }
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        half8_t hi, lo;
#pragma unroll
        for (int ta = 0; ta < 2; ++ta) {
#pragma unroll
            for (int r = 0; r < 4; r += 2) {   // two at a time: packed conversions, mixed-precision subtractions
                const float t0 = t1[ta][tb][r], t1v = t1[ta][tb][r + 1];
                const half2_t h = half2_t{(half_t)t0, (half_t)t1v};
                // t - hi (exact in fp32) as one mixed-precision operation per value, reading hi from its half of
                // the packed register (the compiler converts back and subtracts: two operations)
                float l0, l1;
                asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(l0) : "v"(h), "v"(t0));
                asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(l1) : "v"(h), "v"(t1v));
                const half2_t l = half2_t{(half_t)l0, (half_t)l1};
                hi[4 * ta + r] = h[0];
                hi[4 * ta + r + 1] = h[1];
                lo[4 * ta + r] = l[0];
                lo[4 * ta + r + 1] = l[1];
            }
        }
#pragma unroll
        for (int ta = 0; ta < 2; ++ta) {
            float4_t acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(hi, __builtin_bit_cast(half8_t, H.h2[ta]), zero, 0, 0, 0);
            out[tb][ta] = __builtin_amdgcn_mfma_f32_16x16x32_f16(lo, __builtin_bit_cast(half8_t, H.h2[ta]), acc, 0, 0, 0);
        }
    }
}

// Element index inside the block of out[tb][ta][0] of lane `lane` (the other three follow it).
__device__ __forceinline__ int qp_fwht1024_elem(int lane, int tb, int ta) {
    return 32 * (16 * ta + (lane & 15)) + 16 * tb + 4 * (lane >> 4);
}

// Four transformed values rounded to fp16 (the scale is already in), as two dwords.
__device__ __forceinline__ uint2 qp_fwht1024_pack(const float4_t &v) {
    const half2_t a = half2_t{(half_t)v[0], (half_t)v[1]}, b = half2_t{(half_t)v[2], (half_t)v[3]};
    return uint2{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b)};
}

// ------------------------------------------------------------------ blocks of 2048 .. 8192 on the matrix cores
// A block of 1024 W is W chunks of 1024 (H_{1024 W} = H_W (x) H_1024): W wavefronts transform a chunk each
// (qp_fwht1024_run), park the fp32 results in LDS, and after a barrier 256 threads run the log2 W butterfly
// stages across the chunks, scale by 1 / sqrt(W), round to fp16 and hand out 8 bytes at a time.
// The parking room: QP_FWHT_EX_FLOATS(W) floats, a chunk's element e at e + (e >> 5) * 4 of its 1152 (one
// 16-byte piece of padding per 32 floats keeps the 16-byte writes of a wavefront - rows of 32 floats apart -
// off each other's banks).
#define QP_FWHT_EX_CHUNK 1152
#define QP_FWHT_EX_FLOATS(W) ((W) * QP_FWHT_EX_CHUNK)
__device__ __forceinline__ int qp_fwht_ex_index(int chunk, int e) { return chunk * QP_FWHT_EX_CHUNK + e + ((e >> 5) << 2); }

__device__ __forceinline__ void qp_fwht_park(float *ex, int chunk, int lane, const float4_t (&o)[2][2]) {
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
            *reinterpret_cast<float4_t *>(ex + qp_fwht_ex_index(chunk, qp_fwht1024_elem(lane, tb, ta))) = o[tb][ta];
}

// Thread t (0 .. 255) finishes elements 4 t .. 4 t + 3 of every chunk; store(index in the block, 8 bytes).
// scale = 32 / sqrt(1024 W), the part of the normalisation that the chunks do not carry yet; the product is
// rounded to fp32 and then to fp16, two roundings, always (see qp_scale_round).
template <int W, class Store>
__device__ __forceinline__ void qp_fwht_cross(int t, const float *ex, float scale, Store store) {
    float4_t v[W];
#pragma unroll
    for (int c = 0; c < W; ++c) v[c] = *reinterpret_cast<const float4_t *>(ex + qp_fwht_ex_index(c, 4 * t));
#pragma unroll
    for (int h = 1; h < W; h <<= 1)
#pragma unroll
        for (int c = 0; c < W; ++c)
            if ((c & h) == 0) {
                const float4_t a = v[c], b = v[c + h];
                v[c] = a + b;
                v[c + h] = a - b;
            }
#pragma unroll
    for (int c = 0; c < W; ++c) {
        const half2_t lo = half2_t{qp_scale_round(v[c][0], scale), qp_scale_round(v[c][1], scale)};
        const half2_t hi = half2_t{qp_scale_round(v[c][2], scale), qp_scale_round(v[c][3], scale)};
        store(1024 * c + 4 * t, uint2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)});
    }
}
