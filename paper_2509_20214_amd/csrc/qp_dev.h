// Device-side helpers shared by the gfx950 kernels: layout addressing, per-scheme
// traits and the register-level decode of 8 consecutive weights.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qp.h"

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// What a kernel needs to know about a layer (passed by value).
struct QpW {
    const uint8_t *codes;
    const uint16_t *lut;
    const uint16_t *scales;
    int32_t M, N;
    int64_t row_stride;  // canonical layout only
    int32_t layout;      // qp_layout
    int32_t nbc;         // N / 1024, column blocks per block row (native layout)
    int32_t tlut_bits;   // QP_TCQH: log2 entries of the small table
};

// Compile-time facts about a (scheme, code_bits) pair.
// For QP_TCQHH (half-TCQ) the per-span figures are those of the first half (CB bits per
// step); the second half has CB + 1 bits per step: 16 bytes more per span, one piece more.
template <int S, int CB>
struct QpTraits {
    static constexpr int V = (S == QP_VQ || S == QP_TCQH || S == QP_TCQHH) ? 2 : 1;
    static constexpr int BITS8 = 8 * CB / V;           // stream bits that 8 weights advance
    static constexpr int SPAN = 32 * CB / V;           // bytes of a 256-weight span
    static constexpr int PIECES = SPAN / 16;           // 16-byte pieces per span
    // QP_TCQH: the small table has 2^9 pairs up to 4 bits per weight, 2^10 at 4.5, 2^11 at 5
    // half-TCQ takes the table of its higher bitwidth (App. C.3.2)
    static constexpr int TOP = (S == QP_TCQHH) ? CB + 1 : CB;
    static constexpr bool HYBRID = (S == QP_TCQH || S == QP_TCQHH);
    static constexpr int TLUT_BITS = !HYBRID ? 0 : (TOP <= 8) ? 9 : (TOP == 9) ? 10 : 11;
    static constexpr int LUT_HALVES = (S == QP_TCQ) ? 65536 : HYBRID ? (2 << TLUT_BITS) : (1 << CB) * V;
    static constexpr int BLOCK_BYTES = 64 * SPAN;      // one 16 x 1024 native block
};

// Address of the aligned dword that holds canonical byte `byte_off` of row `row`.
template <int SPAN>
__device__ __forceinline__ const uint32_t *qp_dword_ptr(const QpW &w, int row, int byte_off) {
    if (w.layout == QP_LAYOUT_CANONICAL)
        return reinterpret_cast<const uint32_t *>(w.codes + (int64_t)row * w.row_stride + byte_off);
    int span = byte_off / SPAN;
    int beta = byte_off - span * SPAN;
    int C = span >> 2, g = span & 3, i = row & 15, R = row >> 4;
    int64_t blk = (int64_t)R * w.nbc + C;
    return reinterpret_cast<const uint32_t *>(w.codes + blk * (64 * SPAN) +
                                              ((((beta >> 4) * 64 + g * 16 + i) << 4) + (beta & 15)));
}

// Half-TCQ: address of byte `byte` (a multiple of 4) of 256-weight tile `tile` of row `row`.
// Tiles of the first half (tile < N/512) hold 16 CB bytes, the others 16 (CB + 1).  Native
// layout: a block row is N/2048 blocks of the first kind followed by N/2048 of the second.
template <int CB>
__device__ __forceinline__ const uint32_t *qp_hh_dword_ptr(const QpW &w, int row, int tile, int byte) {
    const int th = w.N >> 9;   // tiles per half
    const bool hi = tile >= th;
    if (w.layout == QP_LAYOUT_CANONICAL) {
        const int64_t off = hi ? (int64_t)th * (16 * CB) + (int64_t)(tile - th) * (16 * (CB + 1))
                               : (int64_t)tile * (16 * CB);
        return reinterpret_cast<const uint32_t *>(w.codes + (int64_t)row * w.row_stride + off + byte);
    }
    const int C = tile >> 2, g = tile & 3, i = row & 15, R = row >> 4, h = w.nbc >> 1;
    const int64_t base = (int64_t)R * h * (1024 * (2 * CB + 1)) +
                         (hi ? (int64_t)h * (1024 * CB) + (int64_t)(C - h) * (1024 * (CB + 1)) : (int64_t)C * (1024 * CB));
    return reinterpret_cast<const uint32_t *>(w.codes + base + ((((byte >> 4) * 64 + g * 16 + i) << 4) + (byte & 15)));
}

// The 64 stream bits that start at the first bit of weight group `grp` (8 weights)
// of row `row`.  For the trellis the second dword wraps inside the 256-weight tile.
template <int S, int CB>
__device__ __forceinline__ uint64_t qp_group_bits(const QpW &w, int row, int grp) {
    using T = QpTraits<S, CB>;
    int d0, d1, r;
    if (S == QP_TCQ) {
        int tile = grp >> 5, u = grp & 31;
        int off = u * T::BITS8;
        r = off & 31;
        int q0 = off >> 5;
        int q1 = (q0 + 1 == T::SPAN / 4) ? 0 : q0 + 1;
        d0 = tile * (T::SPAN / 4) + q0;
        d1 = tile * (T::SPAN / 4) + q1;
    } else {
        int off = grp * T::BITS8;
        r = off & 31;
        d0 = off >> 5;
        // The next dword is read only when the group's BITS8 bits reach into it.  It then holds at
        // least one bit of the row, so it lies inside the row's bytes rounded up to a dword, which
        // the row stride (a multiple of 16, at least the row's bytes rounded up) covers - also when a
        // row of 5- or 7-bit codes ends in the middle of a byte.
        d1 = (r + T::BITS8 > 32) ? d0 + 1 : d0;
    }
    uint32_t lo = *qp_dword_ptr<T::SPAN>(w, row, d0 * 4);
    uint32_t hi = *qp_dword_ptr<T::SPAN>(w, row, d1 * 4);
    return ((((uint64_t)hi) << 32) | lo) >> r;
}

// Decode the 8 weights whose codes start at bit 0 of `bits`.  `lut` is the LDS copy
// of the table.  Every output is a bit copy of a table entry.
template <int S, int CB>
__device__ __forceinline__ void qp_decode8(uint64_t bits, const uint16_t *lut, uint16_t (&w)[8]) {
    if (S == QP_SQ) {
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = lut[(uint32_t)(bits >> (CB * e)) & ((1u << CB) - 1u)];
    } else if (S == QP_VQ) {
        const uint32_t *lut2 = reinterpret_cast<const uint32_t *>(lut);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t p = lut2[(uint32_t)(bits >> (CB * c)) & ((1u << CB) - 1u)];
            w[2 * c] = (uint16_t)p;
            w[2 * c + 1] = (uint16_t)(p >> 16);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = lut[(uint32_t)(bits >> (CB * e)) & 0xffffu];
    }
}

// Entry of the hybrid computed code book for a 16-bit trellis state (Appendix C.3.1,
// "Codebook construction"): h = x (x + 1); the tb bits of h below bit 15 index the small
// table (half2 entries), bit 15 of h negates component 0 - the low half, whose sign bit is
// bit 15 of the dword as well.
__device__ __forceinline__ uint32_t qp_hybrid_entry(uint32_t state, const uint32_t *tlut2, int tb) {
    const uint32_t h = state * (state + 1u);
    const uint32_t idx = (h >> (15 - tb)) & ((1u << tb) - 1u);
    return tlut2[idx] ^ (h & 0x8000u);
}

// 8 consecutive weights (group `grp`) of row `row`, any layout, any scheme.
template <int S, int CB>
__device__ __forceinline__ void qp_group_decode(const QpW &w, int row, int grp, const uint16_t *lut,
                                                uint16_t (&v)[8]) {
    if constexpr (S == QP_TCQHH) {
        const int tile = grp >> 5, u = grp & 31;
        const int cb = CB + ((tile >= (w.N >> 9)) ? 1 : 0);   // bits per step of this tile's half
        const int span4 = 4 * cb;                             // dwords per tile
        const uint32_t *lut2 = reinterpret_cast<const uint32_t *>(lut);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bit = (4 * u + c) * cb;
            const int d0 = bit >> 5, r = bit & 31;
            const int d1 = (d0 + 1 == span4) ? 0 : d0 + 1;   // tail-biting wrap
            const uint32_t lo = *qp_hh_dword_ptr<CB>(w, row, tile, d0 * 4);
            const uint32_t hi = *qp_hh_dword_ptr<CB>(w, row, tile, d1 * 4);
            const uint32_t state = (uint32_t)(((((uint64_t)hi) << 32) | lo) >> r) & 0xffffu;
            const uint32_t e = qp_hybrid_entry(state, lut2, w.tlut_bits);
            v[2 * c] = (uint16_t)e;
            v[2 * c + 1] = (uint16_t)(e >> 16);
        }
    } else if constexpr (S == QP_TCQH) {
        using T = QpTraits<S, CB>;
        const int tile = grp >> 5, u = grp & 31;
        const uint32_t *lut2 = reinterpret_cast<const uint32_t *>(lut);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bit = (4 * u + c) * CB;            // step 4u+c of the tile, CB bits per step
            const int d0 = bit >> 5, r = bit & 31;
            const int d1 = (d0 + 1 == T::SPAN / 4) ? 0 : d0 + 1;   // tail-biting wrap
            const uint32_t lo = *qp_dword_ptr<T::SPAN>(w, row, tile * T::SPAN + d0 * 4);
            const uint32_t hi = *qp_dword_ptr<T::SPAN>(w, row, tile * T::SPAN + d1 * 4);
            const uint32_t state = (uint32_t)(((((uint64_t)hi) << 32) | lo) >> r) & 0xffffu;
            const uint32_t e = qp_hybrid_entry(state, lut2, w.tlut_bits);
            v[2 * c] = (uint16_t)e;
            v[2 * c + 1] = (uint16_t)(e >> 16);
        }
    } else {
        qp_decode8<S, CB>(qp_group_bits<S, CB>(w, row, grp), lut, v);
    }
}

// Copy the table into LDS with all threads of the workgroup (caller synchronises).
template <int HALVES>
__device__ __forceinline__ void qp_stage_lut(const uint16_t *g, uint16_t *s) {
    if (HALVES >= 8 * 64) {
        const u32x4_t *g4 = reinterpret_cast<const u32x4_t *>(g);
        u32x4_t *s4 = reinterpret_cast<u32x4_t *>(s);
        for (int i = threadIdx.x; i < HALVES / 8; i += blockDim.x) s4[i] = g4[i];
    } else {
        const uint32_t *g2 = reinterpret_cast<const uint32_t *>(g);
        uint32_t *s2 = reinterpret_cast<uint32_t *>(s);
        for (int i = threadIdx.x; i < HALVES / 2; i += blockDim.x) s2[i] = g2[i];
    }
}

__device__ __forceinline__ float qp_half_bits_to_float(uint16_t h) {
    return (float)__builtin_bit_cast(half_t, h);
}

// Dispatch a (scheme, code_bits) pair known at run time to a template.
#ifdef QP_DEV_SUBSET  // development builds only: a few schemes, for short compile times
#define QP_DISPATCH_SCHEME(scheme, cb, CALL)                                          \
    do {                                                                              \
        if ((scheme) == QP_SQ && (cb) == 4) { CALL(QP_SQ, 4); }                       \
        else if ((scheme) == QP_VQ && (cb) == 5) { CALL(QP_VQ, 5); }                  \
        else if ((scheme) == QP_VQ && (cb) == 7) { CALL(QP_VQ, 7); }                  \
        else if ((scheme) == QP_TCQH && (cb) == 4) { CALL(QP_TCQH, 4); }              \
        else if ((scheme) == QP_TCQH && (cb) == 8) { CALL(QP_TCQH, 8); }              \
        else return QP_ERR_UNSUPPORTED;                                               \
    } while (0)
#else
#define QP_DISPATCH_SCHEME(scheme, cb, CALL)                                          \
    do {                                                                              \
        if ((scheme) == QP_SQ && (cb) == 4) { CALL(QP_SQ, 4); }                       \
        else if ((scheme) == QP_VQ && (cb) == 5) { CALL(QP_VQ, 5); }                  \
        else if ((scheme) == QP_VQ && (cb) == 7) { CALL(QP_VQ, 7); }                  \
        else if ((scheme) == QP_TCQ && (cb) == 2) { CALL(QP_TCQ, 2); }                \
        else if ((scheme) == QP_TCQ && (cb) == 3) { CALL(QP_TCQ, 3); }                \
        else if ((scheme) == QP_TCQ && (cb) == 4) { CALL(QP_TCQ, 4); }                \
        else if ((scheme) == QP_TCQH && (cb) == 3) { CALL(QP_TCQH, 3); }              \
        else if ((scheme) == QP_TCQH && (cb) == 4) { CALL(QP_TCQH, 4); }              \
        else if ((scheme) == QP_TCQH && (cb) == 5) { CALL(QP_TCQH, 5); }              \
        else if ((scheme) == QP_TCQH && (cb) == 6) { CALL(QP_TCQH, 6); }              \
        else if ((scheme) == QP_TCQH && (cb) == 7) { CALL(QP_TCQH, 7); }              \
        else if ((scheme) == QP_TCQH && (cb) == 8) { CALL(QP_TCQH, 8); }              \
        else if ((scheme) == QP_TCQH && (cb) == 9) { CALL(QP_TCQH, 9); }              \
        else if ((scheme) == QP_TCQH && (cb) == 10) { CALL(QP_TCQH, 10); }            \
        else if ((scheme) == QP_TCQHH && (cb) == 3) { CALL(QP_TCQHH, 3); }            \
        else if ((scheme) == QP_TCQHH && (cb) == 4) { CALL(QP_TCQHH, 4); }            \
        else if ((scheme) == QP_TCQHH && (cb) == 5) { CALL(QP_TCQHH, 5); }            \
        else if ((scheme) == QP_TCQHH && (cb) == 6) { CALL(QP_TCQHH, 6); }            \
        else if ((scheme) == QP_TCQHH && (cb) == 7) { CALL(QP_TCQHH, 7); }            \
        else if ((scheme) == QP_TCQHH && (cb) == 8) { CALL(QP_TCQHH, 8); }            \
        else if ((scheme) == QP_TCQHH && (cb) == 9) { CALL(QP_TCQHH, 9); }            \
        else return QP_ERR_UNSUPPORTED;                                               \
    } while (0)
#endif
