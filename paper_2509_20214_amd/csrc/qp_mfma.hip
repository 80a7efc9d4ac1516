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
// j % TT == t are meaningful.  Summing those columns over t at the end (a DPP fold
// inside each row of 16 lanes) gives the dot products.  TT = 16 / Bp with Bp the batch
// rounded up to a power of two; the TT steps of a fragment share min(TT, 4) accumulators
// through column-masked copies of the fragment.
//
// Table lookups per scheme:
//   SQ 4 bit, VQ 5 and 7 bit : one vector operation per code (two weights): an SDWA shift
//              drops the 8 stream bits that start at the code into byte 1 of a lane's address
//              register; the 256-row table holds one copy of every row per LDS bank, so no
//              two lanes ever collide (QpDecByte).  SQ: a code byte = two 4-bit codes, merged
//              table of half2.  Measured issue cost on this chip, 4 wavefronts per SIMD:
//              2.3 clocks for VOP2 (shift, and, xor), 3.8 for VOP3 / SDWA / DPP forms, so
//              one SDWA per code beats bit-field extract + shift-or (7.6) and shift + and (4.6).
//   VQ 5 bit, small layers, batch 3-4 and 9-16 : 32 entries of half2 = one dword per bank,
//              conflict-free as it is; a private copy per wavefront, no workgroup barrier
//              (QpDecVq5Private).
//              (Keeping the table in a VGPR and fetching it with ds_bpermute saves the
//              AND per code but ran 2x slower: the permute path has a lower rate.)
//   TCQ      : the 2^16-entry fp16 table, 128 KiB of LDS, read with ds_read_u16.
//   TCQH     : computed code book, 1024-entry bank-replicated table (see QpDecTcqh).
//   half-TCQ : TCQH with one 16-byte piece more per lane in the column blocks of the second
//              half of the input channels; a wavefront picks the decoder of its unit's half.
//
// Variants of the same kernel: the activations come row-major from global memory, in
// fragment order from global memory (written that way by the rotation kernel), or - batch 1,
// one Hadamard block of up to 8192 or up to 16 blocks of 1024 - are rotated by the workgroup
// itself into LDS while its first weights are in flight (qp_fwht.h: on the matrix cores; kernel
// instances of their own, so that the plain one does not carry the transform's LDS arrays); for
// the trellis schemes at batch <= 2 a unit can be shared by two wavefronts that decode half of
// its steps each (on request).  The file ends with the dequantize-only
// kernel for the native layout, which reuses the units, loads and decoders.
//
// A workgroup owns a contiguous range of 16-row blocks and walks it in passes of G
// row blocks; the G * (N / 1024) units of a pass are dealt round-robin to the
// wavefronts, each unit's partial sums go to LDS, and after a barrier the workgroup
// adds them up in a fixed order, applies the per-row scale and stores fp16.
#include <type_traits>

#include "qp_internal.h"
#include "qp_fwht.h"

#define QP_NBC_MAX 32  // column blocks of a layer (N <= 32 * 1024)
#ifndef QP_COLMAJOR_MIN_BP
#define QP_COLMAJOR_MIN_BP 4
#endif
// Units per pass: between two passes the workgroup meets at barriers to add up and store, and
// every wavefront starts the next pass in step with the others (all waiting for their loads,
// then all decoding).  The longer a pass, the more the wavefronts drift apart and overlap one
// another's loads with decode; the room for partial sums (16 BP floats per unit) sets the limit.
#ifndef QP_UMAX_SMALL_BATCH
#define QP_UMAX_SMALL_BATCH 128
#endif
// big: beside the 128 KiB table of the V = 1 trellis (32 KiB are left for the partial sums).
#ifndef QP_UMAX_B4
#define QP_UMAX_B4 64
#endif
#ifndef QP_UMAX_B8
#define QP_UMAX_B8 64
#endif
#ifndef QP_UMAX_B16
#define QP_UMAX_B16 64
#endif
#ifdef QP_TRACE   // (the timestamps take 2 KiB of LDS; the 128 KiB trellis table leaves room for 28 units at batch 16 then)
constexpr int qp_umax(int BP, bool big) { return BP == 1 ? QP_UMAX_SMALL_BATCH : (BP <= 4 ? 64 : BP <= 8 ? 32 : 28); }
#else
constexpr int qp_umax(int BP, bool big) {
    return BP == 1 ? QP_UMAX_SMALL_BATCH : BP <= 4 ? (big ? 64 : QP_UMAX_B4) : BP <= 8 ? (big ? 32 : QP_UMAX_B8) : (big ? 32 : QP_UMAX_B16);
}
#endif

#ifdef QP_TRACE  // development builds only: per-wavefront timestamps of the kernel's phases
// Kept in LDS while the kernel runs (a store to global memory would queue behind the weight loads and
// disturb what it measures) and written out by each wavefront when it ends.
__device__ uint64_t *qp_trace_buf;
extern "C" void qp_debug_set_trace(void *p) { (void)hipMemcpyToSymbol(HIP_SYMBOL(qp_trace_buf), &p, sizeof(p)); }
#define QP_TS 20   // slots per wavefront; 16 / 17: the 100 MHz clock that all XCDs share, at start / end
__shared__ uint64_t qp_trace_lds[16 * QP_TS];
// ticks of s_memtime against the 100 MHz constant clock: out[0..1] ticks, out[2..3] 10 ns units
__global__ void k_debug_calibrate(uint64_t *out) {
    const uint64_t t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int i = 0; i < 20000; ++i) __builtin_amdgcn_s_sleep(8);
    const uint64_t t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0) { out[0] = t0; out[1] = t1; out[2] = r0; out[3] = r1; }
}
extern "C" void qp_debug_calibrate(void *out) { hipLaunchKernelGGL(k_debug_calibrate, dim3(1), dim3(64), 0, 0, (uint64_t *)out); }
#define QP_T(slot)                                                                                   \
    do {                                                                                             \
        if ((threadIdx.x & 63) == 0) qp_trace_lds[(threadIdx.x >> 6) * QP_TS + (slot)] =                \
            ((slot) == 16 || (slot) == 17 ? __builtin_amdgcn_s_memrealtime() : __builtin_amdgcn_s_memtime()); \
    } while (0)
#define QP_T_INIT()                                                                                  \
    do {                                                                                             \
        if ((threadIdx.x & 63) < QP_TS) qp_trace_lds[(threadIdx.x >> 6) * QP_TS + (threadIdx.x & 63)] = 0; \
    } while (0)
#define QP_T_FLUSH()                                                                                 \
    do {                                                                                             \
        if ((threadIdx.x & 63) < QP_TS)                                                              \
            qp_trace_buf[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * QP_TS + (threadIdx.x & 63)] = \
                qp_trace_lds[(threadIdx.x >> 6) * QP_TS + (threadIdx.x & 63)];                       \
    } while (0)
#else
#define QP_T(slot)
#define QP_T_INIT()
#define QP_T_FLUSH()
#endif

// ------------------------------------------------------------------ bit fields
// The lane's P pieces seen as one little-endian stream of 128 P bits.  Every index is
// a constant once the step loop is unrolled, so the pieces stay in registers.
template <int P>
__device__ __forceinline__ uint32_t qp_dw(const u32x4_t (&q)[P], int idx) {
    return q[idx >> 2][idx & 3];
}

// 32 stream bits starting at `bitpos` (circular when WRAP; otherwise bits past the end
// of the stream are unspecified).
// PW: pieces that make up the stream (the array may be longer: half-TCQ keeps the units of
// both halves in one array sized for the longer one).
template <int P, bool WRAP, int PW = P>
__device__ __forceinline__ uint32_t qp_bits32(const u32x4_t (&q)[P], int bitpos) {
    const int i0 = bitpos >> 5, r = bitpos & 31;
    if (r == 0) return qp_dw<P>(q, i0);
    const int i1 = WRAP ? ((i0 + 1) % (4 * PW)) : ((i0 + 1 < 4 * PW) ? i0 + 1 : i0);
    return __builtin_amdgcn_alignbit(qp_dw<P>(q, i1), qp_dw<P>(q, i0), r);
}

// (field << LSH) & (mask << LSH) for the nbits-wide field at `bitpos`: one shift and one
// AND when the field sits inside a dword, one funnel shift and one AND when it straddles
// two (a straddling field starts above bit 16 >= LSH, so the funnel can start LSH bits low).
template <int P, bool WRAP, int LSH, int PW = P>
__device__ __forceinline__ uint32_t qp_field_shl(const u32x4_t (&q)[P], int bitpos, int nbits) {
    const int i0 = bitpos >> 5, r = bitpos & 31;
    const uint32_t mask = ((1u << nbits) - 1u) << LSH;
    if (r + nbits <= 32) {
        const uint32_t w = qp_dw<P>(q, i0);
        return ((r >= LSH) ? (w >> (r - LSH)) : (w << (LSH - r))) & mask;
    }
    return qp_bits32<P, WRAP, PW>(q, bitpos - LSH) & mask;
}

// (field << LSH) | orv in two vector operations, v_bfe_u32 + v_lshl_or_b32, with the
// per-lane constant folded into the second (the compiler, left alone, turns the OR into
// a third, separate add).  A field that straddles two dwords costs one funnel shift more.
template <int P, bool WRAP, int LSH>
__device__ __forceinline__ uint32_t qp_field_addr(const u32x4_t (&q)[P], int bitpos, int nbits, uint32_t orv) {
    const int i0 = bitpos >> 5, r = bitpos & 31;
    uint32_t w, idx, a;
    int off;
    if (r + nbits <= 32) {
        w = qp_dw<P>(q, i0);
        off = r;
    } else {
        w = qp_bits32<P, WRAP>(q, bitpos);
        off = 0;
    }
    asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(idx) : "v"(w), "n"(off), "n"(nbits));
    asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(a) : "v"(idx), "n"(LSH), "v"(orv));
    return a;
}

// ------------------------------------------------------------------ per-scheme decode
template <int S, int CB>
struct QpDec;

// Uniform (wave-wide) reads of the table's source go through the scalar cache: they do
// not queue behind the vector loads of the weight stream.
typedef const uint32_t __attribute__((address_space(4))) qp_cu32;
__device__ __forceinline__ qp_cu32 *qp_scalar_ptr(const void *p) {
    return (qp_cu32 *)(uintptr_t)p;
}

// Copy `NQ` 16-byte pieces of the table's source into LDS through scalar registers
// (lane 0 of the calling wavefront writes them).
template <int NQ>
__device__ __forceinline__ void qp_scalar_to_lds(qp_cu32 *src, u32x4_t *dst) {
    u32x4_t v[NQ];
#pragma unroll
    for (int k = 0; k < NQ; ++k) v[k] = u32x4_t{src[4 * k], src[4 * k + 1], src[4 * k + 2], src[4 * k + 3]};
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int k = 0; k < NQ; ++k) dst[k] = v[k];
    }
}

// ---- byte-window decoders (SQ 4 bit, VQ 5 and 7 bit) ---------------------------------------
// A code of at most 8 bits costs ONE vector operation: an SDWA shift (or move) drops the 8
// stream bits that start at the code's first bit into byte 1 of an address register whose
// byte 0 holds 4 (lane % 32) for good.  The table therefore has 256 rows of 256 bytes, row b
// holding 32 copies (one per LDS bank, so lookups never collide) of the entry of window b;
// window bits above the code belong to the next code and are ignored by replicating the
// entry over them (row b = entry b mod 2^CB).  The upper half of every row is unused.
// The address registers are written read-modify-write, so a lane keeps eight of them.
struct QpLane8 {
    uint32_t a[8];
};

template <int SEL>
__device__ __forceinline__ void qp_byte1_from_byte(uint32_t &a, uint32_t w) {
    if constexpr (SEL == 0) asm("v_mov_b32_sdwa %0, %1 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0" : "+v"(a) : "v"(w));
    else if constexpr (SEL == 1) asm("v_mov_b32_sdwa %0, %1 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1" : "+v"(a) : "v"(w));
    else if constexpr (SEL == 2) asm("v_mov_b32_sdwa %0, %1 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2" : "+v"(a) : "v"(w));
    else asm("v_mov_b32_sdwa %0, %1 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3" : "+v"(a) : "v"(w));
}

// byte 1 of `a` <- stream bits [BITPOS, BITPOS + 8) (bits past the lane's stream read as anything)
template <int P, int BITPOS, int NBITS>
__device__ __forceinline__ void qp_window8(const u32x4_t (&q)[P], uint32_t &a) {
    constexpr int i0 = BITPOS >> 5, r = BITPOS & 31;
    if constexpr (r + NBITS <= 32) {
        const uint32_t w = qp_dw<P>(q, i0);
        if constexpr ((r & 7) == 0) {
            qp_byte1_from_byte<r / 8>(a, w);
        } else {
            // the shift amount sits in a scalar register: SDWA encodings take no constants
            asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
                : "+v"(a)
                : "s"(r), "v"(w));
        }
    } else {
        const uint32_t w = qp_bits32<P, false>(q, BITPOS);
        qp_byte1_from_byte<0>(a, w);
    }
}

template <int S, int CB>
struct QpDecByte {
    static constexpr bool BYTE_WINDOW = true;
    static constexpr int TAB_BYTES = 65536;
    static constexpr int SRC_BYTES = (S == QP_SQ) ? 32 : (4 << CB);   // the table's source in global memory
    typedef QpLane8 Lane;
    static constexpr bool DIRECT = (S != QP_SQ);
    // Vector codes: every thread fetches the code book entries that its table rows are made of itself, ahead of
    // everything else (the code book - 128 or 512 bytes - is hot in L2 after the first workgroup): no staging in
    // LDS, no barrier in front of the build (3.5 bit 1024x4096 3.91 -> 3.55 us, 4096x4096 4.23 -> 4.17 us, the step
    // of 4096x14336 8.38 -> 8.31 us).  Scalar codes (a row = two entries of a 32-byte table) keep the staged
    // form: 32 bytes into scalar registers as the very first thing a kernel does - the scalar path does not queue
    // behind the vector loads of the weight stream -, lane 0 writes them to LDS, a barrier, then the build (with
    // two 2-byte fetches per row instead: 4096x4096 3.95 -> 4.30 us).
    static constexpr int NQ = 2;
    struct PreStaged { u32x4_t src[NQ]; };
    struct PreDirect { uint32_t v[4]; };   // the row's entry for idx = thread + k * workgroup size, row idx >> 2
    typedef std::conditional_t<DIRECT, PreDirect, PreStaged> Pre;
    static __device__ __forceinline__ Pre pre(const uint16_t *g, int wgt = (int)blockDim.x) {
        Pre p;
        if constexpr (DIRECT) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int idx = threadIdx.x + k * wgt, b = idx >> 2;
                p.v[k] = idx < 1024 ? reinterpret_cast<const uint32_t *>(g)[b & ((1 << CB) - 1)] : 0u;
            }
        } else {
            qp_cu32 *s = qp_scalar_ptr(g);
#pragma unroll
            for (int k = 0; k < NQ; ++k) p.src[k] = u32x4_t{s[4 * k], s[4 * k + 1], s[4 * k + 2], s[4 * k + 3]};
        }
        return p;
    }
    static __device__ __forceinline__ Lane lane_const() {
        Lane l;
#pragma unroll
        for (int k = 0; k < 8; ++k) l.a[k] = (threadIdx.x & 31u) << 2;
        return l;
    }
    static __device__ __forceinline__ void early(uint8_t *tab, uint16_t *small, const uint16_t *g) { build(tab, small, pre(g)); }
    // every thread writes 32 bytes of a row
    static __device__ __forceinline__ void build(uint8_t *tab, uint16_t *small, const Pre &p, int wgt = (int)blockDim.x) {
        if constexpr (!DIRECT) {
            if (threadIdx.x == 0) {
#pragma unroll
                for (int k = 0; k < NQ; ++k) reinterpret_cast<u32x4_t *>(small)[k] = p.src[k];
            }
            QP_T(11);
            __syncthreads();
        }
        QP_T(12);
        u32x4_t *t4 = reinterpret_cast<u32x4_t *>(tab);
#pragma unroll
        for (int k = 0; k < 4; ++k) {          // (a workgroup has at least 256 threads)
            const int idx = threadIdx.x + k * wgt;
            if (idx < 1024) {
                const int b = idx >> 2, part = idx & 3;
                uint32_t v;
                if constexpr (DIRECT) v = p.v[k];
                else v = (uint32_t)small[b & 15] | ((uint32_t)small[b >> 4] << 16);   // two weights per code byte
                const u32x4_t v4 = u32x4_t{v, v, v, v};
                const int flip = (idx >> 3) & 1;   // neighbouring rows start on different banks
                t4[b * 16 + part * 2 + flip] = v4;
                t4[b * 16 + part * 2 + (flip ^ 1)] = v4;
            }
        }
        QP_T(15);
        __syncthreads();
    }
    template <int P, int SI>
    static __device__ __forceinline__ half8_t step_at(const u32x4_t (&q)[P], const uint8_t *tab, Lane &l) {
        constexpr int CODE = (S == QP_SQ) ? 8 : CB;   // stream bits per lookup (two weights)
        uint32_t r[4];
        qp_window8<P, 4 * CODE * SI + 0 * CODE, CODE>(q, l.a[4 * (SI & 1) + 0]);
        qp_window8<P, 4 * CODE * SI + 1 * CODE, CODE>(q, l.a[4 * (SI & 1) + 1]);
        qp_window8<P, 4 * CODE * SI + 2 * CODE, CODE>(q, l.a[4 * (SI & 1) + 2]);
        qp_window8<P, 4 * CODE * SI + 3 * CODE, CODE>(q, l.a[4 * (SI & 1) + 3]);
#pragma unroll
        for (int c = 0; c < 4; ++c) r[c] = *reinterpret_cast<const uint32_t *>(tab + l.a[4 * (SI & 1) + c]);
        return __builtin_bit_cast(half8_t, u32x4_t{r[0], r[1], r[2], r[3]});
    }
};
template <> struct QpDec<QP_SQ, 4> : QpDecByte<QP_SQ, 4> {};
#ifdef QP_VQ5_BYTE_WINDOW   // (development builds: the one-code-per-lookup form, for comparison)
template <> struct QpDec<QP_VQ, 5> : QpDecByte<QP_VQ, 5> {};
#endif
template <> struct QpDec<QP_VQ, 7> : QpDecByte<QP_VQ, 7> {};

// VQ 5 bit, two codes per lookup: the 10 stream bits of two neighbouring codes index a table of 1024
// entries of 8 bytes (the four weights of the two codes), one ds_read_b64 per four weights instead of two
// ds_read_b32 - a decode step is two shifts, two and-ors and two lookups where the byte-window form has
// four SDWA operations and four lookups.  64 KiB hold eight copies of the table, copy lane % 8 at
// (index << 6) | (lane % 8) << 3: lanes of different copies never share a bank.  An 8-byte lookup is served
// 32 lanes at a time, 64 dwords through 32 banks: two cycles when every pair of banks serves exactly two
// lanes.  Here the four lanes of such a half that share a copy fall on one of the copy's two bank pairs by
// the parity of their index, and the half takes as long as the fullest pair - 3.1 cycles on average
// (measured: 6.2 LDS cycles per 64-lane lookup where 4 is the least).  LSH = 7: sixteen copies in 128 KiB, copy
// lane % 16 at (index << 7) | (lane % 16) << 3 - two lanes per copy and half, one bank pair per copy: always
// the two cycles (measured 4.5 per lookup).  Writing 128 KiB costs the smallest layers more than the
// collisions do (4096x4096 3.77 -> 3.88 us, and the in-kernel rotation has no room beside it); layers of 13 to
// 16 units per workgroup gain on some machines and lose on others (4096x14336 6.66 -> 6.50 us and
// 6.77 -> 6.89 us), larger ones gain everywhere at batch 1 - 2 (10240x8192 8.34 -> 8.01 and 9.11 -> 8.78 us,
// 57344x8192 37.1 -> 32.8 us, batch 2 39.5 -> 37.5; 8192x28672 20.7 -> 19.9, batch 2 22.0 -> 20.4) and are
// unchanged at batch 8 - 16.  The host's rule by units per workgroup is in qp_launch_linear_mfma.
template <int LSH_>
struct QpDecVq5PairT {
    static constexpr bool BYTE_WINDOW = false;
    static constexpr bool AHEAD = true;          // lookups issued ahead of the multiply, like the byte-window decoders
    static constexpr int LSH = LSH_;             // the index sits at bits LSH .. LSH + 9 of a lookup's address
    static constexpr int COPIES = 1 << (LSH - 3);
    static constexpr int TAB_BYTES = 1024 << LSH;
    typedef uint32_t Lane;
    // Every thread fetches the two code book entries that its table entries are made of itself (32 x 4 bytes, hot
    // in L2 after the first workgroup), ahead of everything else: staging the code book in LDS first cost a barrier
    // and an LDS round trip in front of the build (one-launch step of 4096x14336 8.03 -> 7.79 us, 1024x4096
    // 3.71 -> 3.40 us, 4096x4096 3.85 -> 3.80 us, nothing slower).
    struct Pre { uint32_t lo; uint32_t hi[4]; };   // entry idx = thread + k * workgroup size: codes idx & 31 and idx >> 5
    static __device__ __forceinline__ Pre pre(const uint16_t *g, int wgt = (int)blockDim.x) {
        const uint32_t *s = reinterpret_cast<const uint32_t *>(g);
        Pre p;
        p.lo = s[threadIdx.x & 31];                // (the workgroup size is a multiple of 32)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int idx = threadIdx.x + k * wgt;
            p.hi[k] = idx < 1024 ? s[idx >> 5] : 0u;
        }
        return p;
    }
    static __device__ __forceinline__ uint32_t lane_const() { return (threadIdx.x & (uint32_t)(COPIES - 1)) << 3; }
    static __device__ __forceinline__ void early(uint8_t *tab, uint16_t *small, const uint16_t *g) { build(tab, small, pre(g)); }
    static __device__ __forceinline__ void build(uint8_t *tab, uint16_t *, const Pre &p, int wgt = (int)blockDim.x) {
        u32x4_t *t4 = reinterpret_cast<u32x4_t *>(tab);
        QP_T(12);
#pragma unroll
        for (int k = 0; k < 4; ++k) {              // (a workgroup has at least 256 threads)
            const int idx = threadIdx.x + k * wgt;
            if (idx < 1024) {
                const u32x4_t v4 = u32x4_t{p.lo, p.hi[k], p.lo, p.hi[k]};   // first code in the low five bits
                constexpr int NP = COPIES / 2;     // 16-byte pieces per entry
                const int rot = (idx >> (NP == 4 ? 1 : 0)) & (NP - 1);   // neighbouring threads start on different banks
#pragma unroll
                for (int m = 0; m < NP; ++m) t4[idx * NP + ((m + rot) & (NP - 1))] = v4;
            }
        }
        QP_T(15);
        __syncthreads();
    }
    template <int P>
    static __device__ __forceinline__ half8_t step(const u32x4_t (&q)[P], int s, const uint8_t *tab, uint32_t lc,
                                                   const Pre &) {
        uint32_t r[4];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            // 32 stream bits that start LSH bits below the pair: its index then sits at bits LSH .. LSH + 9
            const int from = 20 * s + 10 * c - LSH;
            uint32_t t;
            if (from < 0) {
                t = qp_dw<P>(q, 0) << LSH;
            } else {
                const int i0 = from >> 5, r0 = from & 31;
                if (r0 <= 22 - LSH) t = qp_dw<P>(q, i0) >> r0;
                else t = __builtin_amdgcn_alignbit(qp_dw<P>(q, i0 + 1), qp_dw<P>(q, i0), r0);
            }
            // (the lane's own copy: taking whichever copy the stream bits below the index name - one plain AND -
            // measured 6 % slower, 6.70 -> 7.09 us: collisions are cheap only up to a point)
            const uint32_t a = (t & (1023u << LSH)) | lc;
            const uint2 v = *reinterpret_cast<const uint2 *>(tab + a);
            r[2 * c] = v.x;
            r[2 * c + 1] = v.y;
        }
        return __builtin_bit_cast(half8_t, u32x4_t{r[0], r[1], r[2], r[3]});
    }
};
typedef QpDecVq5PairT<6> QpDecVq5Pair;
typedef QpDecVq5PairT<7> QpDecVq5Pair16;
#ifndef QP_VQ5_BYTE_WINDOW
template <> struct QpDec<QP_VQ, 5> : QpDecVq5Pair {};
#endif

// VQ 5 bit, small layers at some batch sizes: 32 entries of half2 = one dword per LDS bank, conflict-free
// as it is (two lanes either read the same entry or different banks), so every wavefront keeps
// a private copy (16 x 128 bytes), filled from scalar registers once its weight loads are in
// flight.  Two vector operations per code instead of one, but no workgroup barrier in front of
// the decode - which counts when a workgroup only has one unit per wavefront.
struct QpDecVq5Private {
    static constexpr bool BYTE_WINDOW = false;
    static constexpr int TAB_BYTES = 16 * 128;
    typedef uint32_t Lane;
    struct Pre { const uint16_t *g; };
    static __device__ __forceinline__ void early(uint8_t *, uint16_t *, const uint16_t *) {}
    static __device__ __forceinline__ Pre pre(const uint16_t *g, int = 0) { return Pre{g}; }
    static __device__ __forceinline__ void build(uint8_t *tab, uint16_t *, const Pre &p, int = 0) {
        qp_scalar_to_lds<8>(qp_scalar_ptr(p.g), reinterpret_cast<u32x4_t *>(tab) + (threadIdx.x >> 6) * 8);
    }
    static __device__ __forceinline__ uint32_t lane_const() { return (threadIdx.x >> 6) << 7; }
    template <int P>
    static __device__ __forceinline__ half8_t step(const u32x4_t (&q)[P], int s, const uint8_t *tab, uint32_t lc,
                                                   const Pre &) {
        uint32_t r[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t a = qp_field_addr<P, false, 2>(q, 20 * s + 5 * c, 5, lc);
            r[c] = *reinterpret_cast<const uint32_t *>(tab + a);
        }
        return __builtin_bit_cast(half8_t, u32x4_t{r[0], r[1], r[2], r[3]});
    }
};

template <int K>
struct QpDecTcq {
    static constexpr bool BYTE_WINDOW = false;
    static constexpr int TAB_BYTES = 131072;
    static constexpr int PRE = 8;  // 128 KiB / (1024 threads * 16 bytes)
    struct Pre { u32x4_t raw[PRE]; };
    static __device__ __forceinline__ void early(uint8_t *, uint16_t *, const uint16_t *) {}
    static __device__ __forceinline__ Pre pre(const uint16_t *g, int = 0) {  // needs blockDim.x == 1024
        Pre p;
        const u32x4_t *g4 = reinterpret_cast<const u32x4_t *>(g);
#pragma unroll
        for (int k = 0; k < PRE; ++k) p.raw[k] = g4[k * 1024 + threadIdx.x];
        // Hold every wavefront here until all of them have *issued* their share of the
        // table (no wait for the data, hence the bare barrier): the L1 returns in request
        // order, and a table request queued behind another wavefront's cold weight loads
        // would only come back after those.
        __builtin_amdgcn_s_barrier();
        return p;
    }
    static __device__ __forceinline__ void build(uint8_t *tab, uint16_t *, const Pre &p, int = 0) {
        u32x4_t *t4 = reinterpret_cast<u32x4_t *>(tab);
#pragma unroll
        for (int k = 0; k < PRE; ++k) t4[k * 1024 + threadIdx.x] = p.raw[k];
        __syncthreads();
    }
    typedef uint32_t Lane;
    static __device__ __forceinline__ uint32_t lane_const() { return 0; }
    template <int P>
    static __device__ __forceinline__ half8_t step(const u32x4_t (&q)[P], int s, const uint8_t *tab, uint32_t,
                                                   const Pre &) {
        half8_t a;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t ad = qp_field_shl<P, true, 1>(q, (8 * s + e) * K, 16);
            a[e] = __builtin_bit_cast(half_t, *reinterpret_cast<const uint16_t *>(tab + ad));
        }
        return a;
    }
};
// The paper's own trellis (V = 2, computed hybrid code book).  The small table has 2^TB
// half2 entries; the sign flag is bit 15 of h and the index bits sit right below it, so
// bits [15 : 15-TB] of h = x (x + 1) are one (TB+1)-bit index into a table of 2^(TB+1)
// entries in which the upper half is the lower half with component 0 negated.  That table
// fills 64 KiB of LDS with as many copies as fit (entry e, copy c at dword COPIES e + c;
// a lane reads copy l % COPIES): 16, 8 and 4 copies for TB = 9, 10 and 11.  A row of the
// table is then 2^(15 - TB) bytes, which puts the index field of h exactly where the row
// number of the address is: the per-state work is a shift, a 24-bit multiply-add and one
// and-or.  Lanes l and l + 16 of a 32-lane pass share a copy and meet in a bank when their
// rows have the same parity, so a lookup - one per *two* weights - mostly takes two LDS
// cycles per pass instead of one.  (QP_TCQH_TABLE_128K, development builds: 32 copies in
// 128 KiB at TB = 9, one per bank and no collisions, for a bit-field extract and a shift-or
// in place of the and-or; measured slower, the vector pipe being the scarcer one.)
// A lane's state for the V = 2 decoders: the offset of its copy of the table, and (the packed form at 4 bits
// per step) the four addresses that an even decode step worked out for the odd one behind it.  One type for
// every step width, so that the two halves of a half-TCQ layer can share it.
struct QpTcqhLane { uint32_t lc; uint32_t hi[4]; };

template <int TB>
struct QpTcqhPre { uint32_t raw[(1 << TB) / 1024 ? (1 << TB) / 1024 : 1]; };

template <int K, int TB = QpTraits<QP_TCQH, K>::TLUT_BITS>
struct QpDecTcqh {
    static constexpr bool BYTE_WINDOW = false;
    static constexpr int ENTRIES = 2 << TB;
#ifdef QP_TCQH_TABLE_128K
    static constexpr int COPIES = 32768 / ENTRIES;          // 32, 16, 8
    static constexpr int TAB_BYTES = 131072;
#else
    static constexpr int COPIES = 16384 / ENTRIES;          // 16, 8, 4
    static constexpr int TAB_BYTES = 65536;
#endif
    static constexpr int LSH = (COPIES == 32) ? 7 : (COPIES == 16) ? 6 : (COPIES == 8) ? 5 : 4;
    static constexpr int SMALL_BYTES = 4 << TB;             // staging room for the source
    static constexpr int NSRC = (1 << TB) / 1024 ? (1 << TB) / 1024 : 1;   // source dwords per thread
    typedef QpTcqhPre<TB> Pre;
    typedef QpTcqhLane Lane;
    static __device__ __forceinline__ Lane lane_const() { return Lane{(threadIdx.x & (uint32_t)(COPIES - 1)) << 2, {0u, 0u, 0u, 0u}}; }
    static __device__ __forceinline__ void early(uint8_t *, uint16_t *, const uint16_t *) {}
    static __device__ __forceinline__ Pre pre(const uint16_t *g, int = 0) {  // needs blockDim.x == 1024
        Pre p;
#pragma unroll
        // (thread t builds entries t, t + 1024, ... of the table, whose sources are entries (t + 1024 k) mod 2^TB of
        // the small table: it fetches exactly those itself - no staging in LDS, no barrier in front of the build)
        for (int k = 0; k < NSRC; ++k) {
            const int i = (k * 1024 + (int)threadIdx.x) & ((1 << TB) - 1);
            p.raw[k] = reinterpret_cast<const uint32_t *>(g)[i];
        }
        __builtin_amdgcn_s_barrier();   // every wavefront's table request is queued before any weight load
        return p;
    }
    static __device__ __forceinline__ void build(uint8_t *tab, uint16_t *, const Pre &p, int = 0) {
        // Thread t writes all copies of entries t, t + 1024, ...: COPIES / 4 pieces of 16 bytes
        // each, in an order rotated by the lane so that eight neighbouring lanes always cover
        // all 32 banks (a few dozen instructions per thread instead of one per dword).
        u32x4_t *t4 = reinterpret_cast<u32x4_t *>(tab);
        constexpr int NP = COPIES / 4;                          // pieces per entry
        const int rot = (int)(threadIdx.x & 63) >> ((NP == 8) ? 0 : (NP == 4) ? 1 : 2);
#pragma unroll
        for (int m = 0; m < ENTRIES / 1024; ++m) {
            const int e = m * 1024 + (int)threadIdx.x;
            const uint32_t v = p.raw[m & (NSRC - 1)] ^ ((uint32_t)(e >> TB) << 15);
            const u32x4_t v4 = u32x4_t{v, v, v, v};
#pragma unroll
            for (int k = 0; k < NP; ++k) t4[e * NP + ((k + rot) & (NP - 1))] = v4;
        }
        __syncthreads();
    }
    template <int P>
    static __device__ __forceinline__ half8_t step(const u32x4_t (&q)[P], int s, const uint8_t *tab, const Lane &l,
                                                   const Pre &) {
        const uint32_t lc = l.lc;
        uint32_t r[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            // 32 stream bits from the state's first bit on (the stream is K pieces long).  Bits
            // above the 16 of the state are left in: bits 6..15 of x (x + 1), all that is used,
            // depend on the low 16 bits of x only.
            const int bitpos = (4 * s + c) * K, rr = bitpos & 31;
            uint32_t st, h, a;
            // a window that lies inside one dword only needs a plain shift (half the issue cost
            // of the funnel shift)
            if (rr != 0 && rr <= 16) st = qp_dw<P>(q, bitpos >> 5) >> rr;
            else st = qp_bits32<P, true, K>(q, bitpos);
            asm("v_mad_u32_u24 %0, %1, %1, %1" : "=v"(h) : "v"(st));   // x (x + 1) modulo 2^32 (24-bit operands)
#ifdef QP_TCQH_TABLE_128K
            uint32_t idx;
            asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(idx) : "v"(h), "n"(15 - TB), "n"(TB + 1));
            asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(a) : "v"(idx), "n"(LSH), "v"(lc));
#else
            // the index field of h already sits where the row number of the address does
            static_assert(LSH == 15 - TB, "row stride = 2^(15 - TB) bytes");
            // (the lane's own copy; any copy, i.e. h & 0xfffc as one two-operand AND: 8.8 -> 10.4 us on 4096x14336 at 3 bits)
            asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(a) : "v"(h), "s"((ENTRIES - 1) << LSH), "v"(lc));
#endif
            r[c] = *reinterpret_cast<const uint32_t *>(tab + a);
        }
        return __builtin_bit_cast(half8_t, u32x4_t{r[0], r[1], r[2], r[3]});
    }
};
// 4 and 8 bits per step (2 and 4 bits per weight): states 16 / K steps apart start 16 bits apart, so one 32-bit
// window of the stream holds TWO states in its two halves, and one packed 16-bit multiply-add hashes both -
// h = x (x + 1) is only needed modulo 2^16.  Per pair of states: one funnel shift (none where the window is a
// dword of the stream), one v_pk_mad_u16, one and-or for the low half's address, a shift and an and-or for the
// high half's: five vector operations where the plain form has six.  At 4 bits per step the two states of a
// window belong to two consecutive decode steps (the even step hashes for both and parks the odd step's four
// addresses in the lane's state), at 8 bits to the same step.
template <int K, int TB = QpTraits<QP_TCQH, K>::TLUT_BITS>
struct QpDecTcqhPacked : QpDecTcqh<K, TB> {
    static_assert(K == 4 || K == 8, "two states per 32-bit window");
    typedef QpDecTcqh<K, TB> Base;
    typedef typename Base::Pre Pre;
    typedef QpTcqhLane Lane;
    // addresses of the two states in the halves of `win`
    static __device__ __forceinline__ void pair(uint32_t win, uint32_t lc, uint32_t &a_lo, uint32_t &a_hi) {
        static_assert(Base::LSH == 15 - TB, "the index field of the hash is the row number of the address");
        uint32_t h, t;
        asm("v_pk_mad_u16 %0, %1, %1, %1" : "=v"(h) : "v"(win));   // x (x + 1) modulo 2^16 in both halves
        asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(a_lo) : "v"(h), "s"((Base::ENTRIES - 1) << Base::LSH), "v"(lc));
        t = h >> 16;
        asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(a_hi) : "v"(t), "s"((Base::ENTRIES - 1) << Base::LSH), "v"(lc));
    }
    template <int P>
    static __device__ __forceinline__ half8_t step(const u32x4_t (&q)[P], int s, const uint8_t *tab, Lane &l, const Pre &) {
        uint32_t r[4];
        if constexpr (K == 4) {
            if ((s & 1) == 0) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    uint32_t a;
                    pair(qp_bits32<P, true, K>(q, 16 * s + 4 * c), l.lc, a, l.hi[c]);   // states 4 s + c and 4 (s + 1) + c
                    r[c] = *reinterpret_cast<const uint32_t *>(tab + a);
                }
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) r[c] = *reinterpret_cast<const uint32_t *>(tab + l.hi[c]);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                uint32_t a, b;
                pair(qp_bits32<P, true, K>(q, 32 * s + 8 * c), l.lc, a, b);   // states 4 s + c and 4 s + c + 2
                r[c] = *reinterpret_cast<const uint32_t *>(tab + a);
                r[c + 2] = *reinterpret_cast<const uint32_t *>(tab + b);
            }
        }
        return __builtin_bit_cast(half8_t, u32x4_t{r[0], r[1], r[2], r[3]});
    }
};
#ifdef QP_TCQH_TABLE_128K
template <> struct QpDec<QP_TCQH, 4> : QpDecTcqh<4> {};
template <> struct QpDec<QP_TCQH, 8> : QpDecTcqh<8> {};
#else
template <> struct QpDec<QP_TCQH, 4> : QpDecTcqhPacked<4> {};
template <> struct QpDec<QP_TCQH, 8> : QpDecTcqhPacked<8> {};
#endif
template <> struct QpDec<QP_TCQH, 3> : QpDecTcqh<3> {};
template <> struct QpDec<QP_TCQH, 5> : QpDecTcqh<5> {};
template <> struct QpDec<QP_TCQH, 6> : QpDecTcqh<6> {};
template <> struct QpDec<QP_TCQH, 7> : QpDecTcqh<7> {};
template <> struct QpDec<QP_TCQH, 9> : QpDecTcqh<9> {};
template <> struct QpDec<QP_TCQH, 10> : QpDecTcqh<10> {};

// Half-TCQ (Section 3.2, App. C.3.2): column blocks of the first half of the input channels
// carry K bits per step, those of the second half K + 1; one table, that of K + 1.
// QpDec<QP_TCQHH, K> is the decoder of the second half (it also builds the table); Lo
// decodes the first half from the same table.
template <int K, int TB> struct QpTcqhPick { typedef QpDecTcqh<K, TB> type; };
#ifndef QP_TCQH_TABLE_128K
template <int TB> struct QpTcqhPick<4, TB> { typedef QpDecTcqhPacked<4, TB> type; };
template <int TB> struct QpTcqhPick<8, TB> { typedef QpDecTcqhPacked<8, TB> type; };
#endif
template <int K>
struct QpDecHalf : QpTcqhPick<K + 1, QpTraits<QP_TCQHH, K>::TLUT_BITS>::type {
    typedef typename QpTcqhPick<K, QpTraits<QP_TCQHH, K>::TLUT_BITS>::type Lo;
};
template <> struct QpDec<QP_TCQHH, 3> : QpDecHalf<3> {};
template <> struct QpDec<QP_TCQHH, 4> : QpDecHalf<4> {};
template <> struct QpDec<QP_TCQHH, 5> : QpDecHalf<5> {};
template <> struct QpDec<QP_TCQHH, 6> : QpDecHalf<6> {};
template <> struct QpDec<QP_TCQHH, 7> : QpDecHalf<7> {};
template <> struct QpDec<QP_TCQHH, 8> : QpDecHalf<8> {};
template <> struct QpDec<QP_TCQHH, 9> : QpDecHalf<9> {};

template <> struct QpDec<QP_TCQ, 2> : QpDecTcq<2> {};
template <> struct QpDec<QP_TCQ, 3> : QpDecTcq<3> {};
template <> struct QpDec<QP_TCQ, 4> : QpDecTcq<4> {};

// Decoders whose workgroup-wide table can be built either before the first loads are issued
// (early) or after (build) define both to do the same thing; the kernel calls exactly one.
// Early delays most loads by the fetch of the table's source, the LDS writes and a barrier; late makes
// every wavefront wait at a barrier until the slowest one has issued its loads.  Measured (SQ 4 bit):
// late wins for workgroups with few units (4096x4096: 5.8 -> 4.4 us), early for many
// (4096x14336: 8.2 vs 9.3 us).
template <class D> struct QpTableMovable { static constexpr bool value = false; };
template <> struct QpTableMovable<QpDec<QP_SQ, 4>> { static constexpr bool value = true; };
template <> struct QpTableMovable<QpDec<QP_VQ, 7>> { static constexpr bool value = true; };
template <> struct QpTableMovable<QpDec<QP_VQ, 5>> { static constexpr bool value = true; };
template <> struct QpTableMovable<QpDecVq5Pair16> { static constexpr bool value = true; };

// ALT selects the second form of a kernel where there is one: two wavefronts per unit for the
// V = 1 and V = 2 trellis; for VQ 5 bit the sixteen-copy table of code pairs at batch 1 - 2 and the
// per-wavefront table at batch 3 - 4.
template <int S, int CB, bool ALT, int BP> struct QpDecSel { typedef QpDec<S, CB> type; };
template <int BP> struct QpDecSel<QP_VQ, 5, true, BP> {
    typedef std::conditional_t<(BP <= 2), QpDecVq5Pair16, QpDecVq5Private> type;
};
constexpr bool qp_alt_splits(int S) { return S == QP_TCQ || S == QP_TCQH; }

// Step SI of a unit with the step index as a compile-time constant (the byte-window decoders
// pick their instruction forms from it).
template <class D, int P, int SI>
__device__ __forceinline__ half8_t qp_step(const u32x4_t (&q)[P], const uint8_t *tab, typename D::Lane &lc,
                                           const typename D::Pre &pre) {
    if constexpr (D::BYTE_WINDOW) return D::template step_at<P, SI>(q, tab, lc);
    else return D::template step<P>(q, SI, tab, lc, pre);
}

// Decoders whose lookups are issued ahead of the multiply: the byte-window ones, and those that say so.
template <class D, class = void> struct QpAhead { static constexpr bool value = D::BYTE_WINDOW; };
template <class D> struct QpAhead<D, decltype((void)D::AHEAD)> { static constexpr bool value = D::AHEAD; };
template <class D> constexpr bool qp_looks_ahead() { return QpAhead<D>::value; }

template <int B, int E, class F>
__device__ __forceinline__ void qp_static_for(F &&f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        qp_static_for<B + 1, E>(f);
    }
}

// ------------------------------------------------------------------ DPP fold
// v + (src shifted towards lane 0 by N lanes inside each row of 16 lanes).
template <int N>
__device__ __forceinline__ float qp_add_row_shl(float v, float src) {
    int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, src), 0x100 + N, 0xf, 0xf, true);
    return v + __builtin_bit_cast(float, moved);
}

template <int TT, int T = 1>
struct QpFold {  // acc[0] + shl1(acc[1]) + ... : lane b*TT of every row ends up with the sum over t
    static __device__ __forceinline__ void run(float4_t &v, const float4_t (&acc)[TT]) {
        if constexpr (T < TT) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = qp_add_row_shl<T>(v[e], acc[T][e]);
            QpFold<TT, T + 1>::run(v, acc);
        }
    }
};

// ------------------------------------------------------------------ the kernel
// One unit's loads: the first PF activation fragments, then P coalesced 128-bit pieces
// of codes.  Straight-line code (no branches) so that the waits the compiler inserts
// later can name exactly the loads they need.
// The P pieces of one unit.  Half-TCQ units of the first half have one piece less: `full`
// (wave-uniform) says whether the last one exists.
// One 16-byte piece of the weight stream: read once, never reused, hence non-temporal (measured
// 5 - 8 % faster than plain loads on large layers; the sc0 policy on top changes nothing).
__device__ __forceinline__ u32x4_t qp_stream_load(const u32x4_t *p) { return __builtin_nontemporal_load(p); }

template <int P, bool OPTIONAL_LAST>
// src: the lane's first piece; ps: distance between its pieces in 16-byte units (64 in the
// native layout, where a piece of all 64 lanes is one contiguous KiB; 1 in the canonical one,
// where the lane's pieces follow each other in its row).
__device__ __forceinline__ void qp_pieces_load(const u32x4_t *src, int ps, bool full, u32x4_t (&q)[P]) {
#ifdef QP_NOLOAD  // development builds only: decode without the weight stream, to time the compute side alone
    {
        const uint32_t h = (uint32_t)(uintptr_t)src * 2654435761u;
#pragma unroll
        for (int p = 0; p < P; ++p) q[p] = u32x4_t{h + p, h ^ (0x9e3779b9u * (p + 1)), h * (2 * p + 3), ~h + 7 * p};
        return;
    }
#endif
#pragma unroll
    for (int p = 0; p < P; ++p) {
        if (OPTIONAL_LAST && p == P - 1) {
            q[p] = u32x4_t{0u, 0u, 0u, 0u};
            if (full) q[p] = qp_stream_load(src + p * ps);
        } else {
            q[p] = qp_stream_load(src + p * ps);
        }
    }
}

// Where a unit's activation fragments are.
// Batch 5 - 16, global memory (QpXBuf): a buffer descriptor over the whole activation array, the
// unit's column block and the fragment number as a wave-uniform byte offset (scalar registers)
// and the lane's own byte offset, which is the same for every fragment, column block and unit -
// one vector register and no vector address arithmetic per load, where a flat 64-bit address
// costs a register pair and an add each.  These kernels sit at the register limit and load 16
// to 32 fragments per unit (fragment-order activations at batch 16: 57344x8192 VQ 5 bit
// 66 -> 57 us, 4096x14336 SQ 18.3 -> 13.9 us); at batch <= 4 there are 2 - 8 loads per unit and
// the flat form (QpXPtr: the lane's own pointer, also used for the copy in LDS that the in-kernel
// rotation leaves) measured the same or better.
struct QpXBuf {
    static constexpr bool TIE_REFILLS = true;
    __amdgpu_buffer_rsrc_t rsrc;
    int soff;      // bytes to the unit's column block
    uint32_t lo;   // the lane's bytes
    int xfs;       // bytes between fragments
    // (Kernels of whole blocks carry these two as constants.  They stay members all the same: without them the
    // register allocator gives the batch-16 kernels 128 registers and spills where it now takes 99 and none -
    // 4-bit scalar 4096x14336 at batch 16 14.9 against 13.9 us.)
    bool tail;     // (wave-uniform) the unit's column block is cut short by N: `keep` applies
    uint32_t keep; // all ones, or zero where the lane's 256 columns lie beyond N
    __device__ __forceinline__ half8_t frag(int n, uint32_t lane_off) const {
#ifdef QP_NOX  // development builds only: no activation loads, to time what they cost
        return __builtin_bit_cast(half8_t, u32x4_t{lane_off, (uint32_t)(soff + xfs * n), 0x3c003c00u, 0x3c003c00u});
#endif
        return __builtin_bit_cast(half8_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_off, soff + xfs * n, 0));
    }
    __device__ __forceinline__ half8_t frag(int n) const { return frag(n, lo); }
};
struct QpXPtr {
    static constexpr bool TIE_REFILLS = false;
    const half_t *p;   // the lane's first fragment of the unit
    uint32_t lo;       // unused (0)
    int xfs;           // halves between fragments
    bool tail;         // (wave-uniform) the unit's column block is cut short by N: `keep` applies
    uint32_t keep;     // all ones, or zero where the lane's 256 columns lie beyond N
    __device__ __forceinline__ half8_t frag(int n, uint32_t) const { return frag(n); }
    __device__ __forceinline__ half8_t frag(int n) const {
#ifdef QP_NOX  // development builds only: no activation loads, to time what they cost
        return __builtin_bit_cast(half8_t, u32x4_t{(uint32_t)(uintptr_t)p, (uint32_t)n, 0x3c003c00u, 0x3c003c00u});
#endif
        return *reinterpret_cast<const half8_t *>(p + xfs * n);
    }
};

template <int P, int PF, bool OPTIONAL_LAST, class XS>
__device__ __forceinline__ void qp_unit_load(const u32x4_t *src, int ps, const XS &xs, bool full,
                                             u32x4_t (&q)[P], half8_t (&xf)[PF]) {
#pragma unroll
    for (int n = 0; n < PF; ++n) xf[n] = xs.frag(n);
    qp_pieces_load<P, OPTIONAL_LAST>(src, ps, full, q);
}

// Two wavefronts per unit (trellis schemes, few units per workgroup): half H decodes steps
// 16 H .. 16 H + 15 and only needs the pieces that hold its windows - those of its own half of
// the stream plus, the windows being 16 bits wide, the piece after it (for the second half: the
// first piece, by tail-biting).  The others stay zero and are never looked at.
// PHASE 0: everything; 1: only the piece that holds the half's first window; 2: the others.
template <int S, int CB, int P, int H, int PHASE = 0>
__device__ __forceinline__ void qp_half_pieces_load(const u32x4_t *src, int ps, u32x4_t (&q)[P]) {
    constexpr int V = QpTraits<S, CB>::V;
    constexpr int ELEMS = 128 / V;                       // windows per half
    constexpr int TOTAL = 128 * P;                       // stream bits of the lane
    constexpr int START = H * ELEMS * CB, END = START + (ELEMS - 1) * CB + 16;   // [START, END)
    constexpr int FIRST = START / 128;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const bool need = (128 * p < END && 128 * p + 128 > START) || (END > TOTAL && 128 * p < END - TOTAL);
        if (PHASE == 1 && p != FIRST) continue;
        if (PHASE == 2 && p == FIRST) continue;
        if (need) q[p] = qp_stream_load(src + p * ps);
        else q[p] = u32x4_t{0u, 0u, 0u, 0u};
    }
}

// Decode and multiply one unit; the lane that owns (rows 4g..4g+3, batch row b) returns
// their partial dot products in v.
// S0, S1: the steps done here (a whole unit, or one half of it when two wavefronts share a
// unit); xf[i] holds fragment S0 / TT + i on entry.
template <class D, int P, int PF, int TT, int S0 = 0, int S1 = 32, class XS>
__device__ __forceinline__ float4_t qp_unit_compute(const u32x4_t (&q)[P], half8_t (&xf)[PF], const XS &xs,
                                                    const uint8_t *tab, typename D::Lane &lc,
                                                    const typename D::Pre &pre) {
    constexpr int N0 = S0 / TT, N1 = S1 / TT;   // fragments N0 .. N1 - 1
#ifdef QP_NODECODE  // development builds only: loads without decode, to time the memory side alone
    {
        uint32_t z = 0;
#ifdef QP_TRACE   // arrival of the first, the middle and the last piece (one load, the scale, was issued after them)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(P) : "memory");
        QP_T(18);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(P - P / 2) : "memory");
        QP_T(19);
        asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
        QP_T(10);
#endif
#pragma unroll
        for (int p = 0; p < P; ++p) z ^= q[p][0] ^ q[p][1] ^ q[p][2] ^ q[p][3];
#pragma unroll
        for (int n = 0; n < PF; ++n) z ^= __builtin_bit_cast(u32x4_t, xf[n])[0];
        return float4_t{(float)z, 0.f, 0.f, 0.f};
    }
#endif
    // NACC accumulators serve the TT steps of a fragment: step t adds into acc[t % NACC]
    // and multiplies with a copy of the fragment in which only the columns of its own
    // group (t / NACC) are kept, the others zeroed.  Column j of acc[a] then holds exactly
    // the steps with t % TT == j % TT (if that is congruent to a; garbage-free zeros
    // otherwise), and far fewer accumulators have to be folded than with one per step.
    constexpr int NACC = (TT < 4) ? TT : 4;
    constexpr int NM = TT / NACC;
    const int lane_t = (int)(threadIdx.x & 15) % TT;
    float4_t acc[NACC];
#pragma unroll
    for (int t = 0; t < NACC; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
    u32x4_t masked[NM];
    uint32_t keep[NM];
    uint32_t xlo = xs.lo, dep = 0;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
        keep[m] = (lane_t / NACC) == m ? 0xffffffffu : 0u;
        asm volatile("" : "+v"(keep[m]));   // stays a register: the compiler would turn the AND back into a select
    }
    // The table lookups of a step are issued DEPTH steps ahead of the matrix instruction that consumes
    // them.  Left to itself the compiler issues the lookups of two steps and waits for them right
    // away; a wavefront that has its SIMD to itself (a workgroup with four units, or the last wavefront
    // of a workgroup to get its data) then sits out the LDS latency once per pair of steps.  Measured on
    // 4096x4096 at 2.5 bits: batch 1 4.19 -> 4.01 us, batch 4 4.60 -> 4.34 us, batch 8 4.38 -> 4.21 us;
    // within 1 % either way on 4096x14336 and larger.  Not at one step per fragment (batch 9 - 16),
    // where the registers do not allow it (spills: 12 -> 51 us).
#ifndef QP_PIPE_DEPTH_BYTE
#define QP_PIPE_DEPTH_BYTE 4
#endif
#ifndef QP_PIPE_DEPTH_TRELLIS
#define QP_PIPE_DEPTH_TRELLIS 0
#endif
    constexpr int DEPTH = (TT == 1) ? 0 : (qp_looks_ahead<D>() ? QP_PIPE_DEPTH_BYTE : QP_PIPE_DEPTH_TRELLIS);
    half8_t pipe[DEPTH > 0 ? DEPTH : 1];
    qp_static_for<0, DEPTH>([&](auto dc) __attribute__((always_inline)) {
        constexpr int d = decltype(dc)::value;
        if constexpr (S0 + d < S1) pipe[d] = qp_step<D, P, S0 + d>(q, tab, lc, pre);
    });
    qp_static_for<S0, S1>([&](auto sc) __attribute__((always_inline)) {
        constexpr int s = decltype(sc)::value;
        constexpr int n = s / TT, t = s % TT;
        if constexpr (t == 0) {
            u32x4_t raw = __builtin_bit_cast(u32x4_t, xf[(n - N0) % PF]);
            if (xs.tail) {   // lane groups beyond N: whatever was fetched for them becomes zero
#pragma unroll
                for (int r = 0; r < 4; ++r) raw[r] &= xs.keep;
            }
            if constexpr (NM == 1) {
                masked[0] = raw;
            } else {
#pragma unroll
                for (int m = 0; m < NM; ++m) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) masked[m][r] = raw[r] & keep[m];   // (an AND issues in 2.3 clocks, a select in 3.8)
                }
            }
            if constexpr (n + PF < N1) {  // the raw fragment is spent: refill its slot
                // One step per fragment (batch 9 - 16): the refill is tied to the previous step's
                // decoded operand.  Left free, the scheduler hoists the refills of many steps to the
                // top of the unit, runs out of registers and spills fragments - and a spill store
                // waits for every load in flight.
                if constexpr (TT == 1 && n > N0 && XS::TIE_REFILLS) asm volatile("" : "+v"(xlo) : "v"(dep));
                xf[(n - N0) % PF] = xs.frag(n + PF, xlo);
            }
        }
        half8_t a;
        if constexpr (DEPTH > 0) {
            a = pipe[(s - S0) % DEPTH];
            if constexpr (s + DEPTH < S1) {
                pipe[(s - S0) % DEPTH] = qp_step<D, P, s + DEPTH>(q, tab, lc, pre);
                __builtin_amdgcn_sched_barrier(0);   // the lookups above stay in front of the multiply below
            }
        } else {
            a = qp_step<D, P, s>(q, tab, lc, pre);
        }
        if constexpr (TT == 1 && XS::TIE_REFILLS) dep = __builtin_bit_cast(u32x4_t, a)[3];
        acc[t % NACC] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, __builtin_bit_cast(half8_t, masked[t / NACC]),
                                                               acc[t % NACC], 0, 0, 0);
#ifdef QP_TRACE
        if constexpr (s == 0) QP_T(3);
        if constexpr (s == 27) QP_T(4);
#endif
    });
    float4_t v = acc[0];
    QpFold<NACC>::run(v, acc);   // lanes with t % NACC == 0 now hold their group's sum
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if constexpr (NM >= 2) v[e] = qp_add_row_shl<NACC>(v[e], v[e]);
        if constexpr (NM >= 4) v[e] = qp_add_row_shl<2 * NACC>(v[e], v[e]);
    }
    return v;
}

// After a pass: wait for every wavefront's partial sums, add them per output in a fixed
// order (column blocks ascending), scale, round once to fp16 and store.
template <int BP>
__device__ __forceinline__ void qp_pass_store(const QpW &w, const float *red, half_t *y, int64_t ldy, int B,
                                              int rb0, int gcount, int nbc, uint16_t scale_first, int wgt) {
    constexpr int LB = (BP == 1) ? 0 : (BP == 2) ? 1 : (BP == 4) ? 2 : (BP == 8) ? 3 : 4;
    __syncthreads();
    QP_T(5);
    for (int o = threadIdx.x; o < (gcount << (4 + LB)); o += wgt) {
        const int i = o & 15, b = (o >> 4) & (BP - 1), slot = o >> (4 + LB);
        if (b < B) {
            const int row = (rb0 + slot) * 16 + i;
            const uint16_t sc = (o == (int)threadIdx.x) ? scale_first : w.scales[row];
            float sum = 0.f;
            const float *r = &red[((slot * nbc) * BP + b) * 16 + i];
            for (int C0 = 0; C0 < nbc; C0 += 8) {  // eight independent LDS reads in flight, fixed order
                float part[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int C = C0 + k;
                    part[k] = r[(C < nbc ? C : nbc - 1) * BP * 16];
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) sum += (C0 + k < nbc) ? part[k] : 0.f;
            }
            y[(int64_t)b * ldy + row] = (half_t)(qp_half_bits_to_float(sc) * sum);
        }
    }
    __syncthreads();
}

// Shapes of the LDS arrays of the fused kernel.
template <class D, int S, int CB, int BP>
struct QpLinLds {
    using T = QpTraits<S, CB>;
    static constexpr int RED_FLOATS = qp_umax(BP, D::TAB_BYTES > 65536) * 16 * BP;
    static constexpr int SMALL_FLOATS = T::HYBRID ? (1 << T::TLUT_BITS) : 0;
    static constexpr int RED = RED_FLOATS > SMALL_FLOATS ? RED_FLOATS : SMALL_FLOATS;
    // in-kernel rotation (batch 1, one Hadamard block of at most 8192): the rotated
    // activations (fp16), and the transform's constant matrices and parked chunks (fp32),
    // which borrow the table's room where that is large enough and still unused
    static constexpr int ROT_MAX = 8192;
    static constexpr int ROT_SCRATCH_FLOATS = 1024 + QP_FWHT_EX_FLOATS(ROT_MAX / 1024);   // constant matrices, parked chunks
    // (not beside the 128 KiB table of the V = 1 trellis: the transform would have to borrow the table's room
    // and run before the table is built - measured no faster than two launches, 8192x8192 23.6 against 20.7 us)
    static constexpr bool ROT = (BP == 1) && D::TAB_BYTES <= 65536;
    // per-wavefront rotation of N / 1024 <= 16 blocks (batch 1): the rotated activations of the whole
    // row; the 128 KiB table leaves no room for that
    static constexpr int ROTM_MAX = 16384;
    static constexpr bool ROTM = (BP == 1) && D::TAB_BYTES <= 65536;
    // every table build of these kernels has a workgroup barrier behind the point where the transform's
    // constants are written - except the per-wavefront table
    static constexpr bool TABLE_HAS_BARRIER = D::TAB_BYTES > 16 * 128;
};

// XL: the activations are rotated here (Section 3.3), by the workgroup itself, into LDS, and
// the B-operand fragments are read from there; otherwise they come from global memory.
// XL == 1: one Hadamard block of 1024 W <= 8192, a chunk of 1024 per wavefront on the matrix cores and
// log2 W butterfly stages across the chunks (qp_fwht_cross).
// XL == 2: N / 1024 <= 16 blocks of 1024 and one row block per workgroup; every wavefront transforms
// the block of its own unit on the matrix cores (qp_fwht1024_run, shared with the stand-alone kernel,
// so the same bits).
// TN: N is not a multiple of 1024 (a kernel of its own: the masks cost the others 2 - 6 %).
template <int S, int CB, int BP, int XL, bool ALT, bool TN = false>
__device__ __forceinline__ void qp_linear_body(const QpW &w, const half_t *x, int B, int64_t ldx, half_t *y,
                                               int64_t ldy, int G, int rb_q, int rb_r, int nbc_magic,
                                               int x_flags, const int8_t *signs, int rot_block, float rot_norm, uint8_t *tab,
                                               float *red, half_t *xr_lds, float *rot_buf) {
    uint32_t *had_lds = reinterpret_cast<uint32_t *>(rot_buf);   // in-kernel rotation: 4 KiB for the transform's constant matrices
    const int x_packed = x_flags & 0xff;   // activations in fragment order
    const int late_max = x_flags >> 8;     // a movable table is built after the first loads up to this many units
    using T = QpTraits<S, CB>;
    using D = typename QpDecSel<S, CB, ALT, BP>::type;
    constexpr bool SPLIT = ALT && qp_alt_splits(S);
    // Half-TCQ: the units of the second half of the column blocks have P pieces and decode
    // with D, those of the first half have P - 1 and decode with D::Lo; both kinds share the
    // piece array, the table and everything else.
    constexpr bool HH = (S == QP_TCQHH);
    constexpr int P = HH ? T::PIECES + 1 : T::PIECES;
    constexpr int LB = (BP == 1) ? 0 : (BP == 2) ? 1 : (BP == 4) ? 2 : (BP == 8) ? 3 : 4;
    // steps per activation fragment; 16 accumulators only where the registers allow it
    constexpr int TTMAX = 16;
    constexpr int TT = (16 / BP < TTMAX) ? 16 / BP : TTMAX;
    constexpr int NXF = 32 / TT;                     // activation fragments per unit
    // SPLIT: a unit is shared by two wavefronts, each decoding 16 of its 32 steps; the work
    // items of a pass are then the half units, item u = 2 * unit + half.
    constexpr int SPL = SPLIT ? 2 : 1;
    static_assert(!SPLIT || (!HH && NXF >= 2 && NXF <= 4), "half units: trellis schemes, batch <= 2");
#ifndef QP_PF_MAX16
#define QP_PF_MAX16 8
#endif
    constexpr int PFMAX = (BP == 16) ? QP_PF_MAX16 : 8;
    constexpr int PF = SPLIT ? NXF / 2 : ((NXF < PFMAX) ? NXF : PFMAX);   // fragments kept in flight
    constexpr int BLK16 = T::BLOCK_BYTES / 16;
    QP_T_INIT();
    QP_T(16);
    QP_T(0);

    // ---- first pass, straight-line up to the first loads ------------------------------
    // The source of a table that the whole workgroup shares is requested here, ahead of every other load
    // (every thread the code book entries of its own table entries; scalar codes through scalar registers);
    // a per-wavefront table only fetches its source here and is written once the weight loads are in
    // flight; the trellis table's source is requested first so that it can be waited for alone.
    // (a table that can be built at either point: late when the workgroup has few units)
    constexpr bool MOVABLE = QpTableMovable<D>::value;
    // (not where the in-kernel rotation's scratch borrows the table's room first)
    constexpr bool MID_BUILD = !MOVABLE &&
                               (S == QP_TCQ || S == QP_TCQH || S == QP_TCQHH);
    const bool table_late = MOVABLE && (rb_q + (rb_r ? 1 : 0)) * w.nbc <= late_max;
    QP_T(13);
    // Threads of the workgroup.  XL == 2 always runs 16 wavefronts, and so do the trellis schemes (the host sets
    // it): a constant there instead of a kernel argument on a cache line of its own, and the rounds "one entry per
    // thread, as many as it takes" of the table build, the transform's constants and the sums become straight-line
    // code.  Taken where it measured faster: XL == 2, and the trellis kernels that rotate one block themselves
    // (hybrid trellis steps 4096x8192 at 2 bits 6.48 -> 6.06 us, 4096x4096 4.79 -> 4.62 us; their other kernels
    // within 3 % either way; 16 wavefronts and the constant for the scalar and vector quantizers at XL == 1, which
    // run 8 to 16: 2.5 bits 4096x4096 4.40 -> 4.29 us but 4096x8192 5.96 -> 6.35 us).
    constexpr bool WG_1024 = XL == 2 || (XL == 1 && (S == QP_TCQH || S == QP_TCQHH));
    const int wgt = WG_1024 ? 1024 : (int)blockDim.x;
    const typename D::Pre pre = D::pre(w.lut, wgt);

    const int nw = wgt >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nbc = w.nbc;
    // balanced contiguous partition of the row blocks over the workgroups: the first rb_r
    // workgroups take rb_q + 1 blocks, the others rb_q
    const int bx = blockIdx.x;
    const int rb_begin = bx * rb_q + (bx < rb_r ? bx : rb_r);
    const int rb_end = rb_begin + rb_q + (bx < rb_r ? 1 : 0);
    const u32x4_t *codes16 = reinterpret_cast<const u32x4_t *>(w.codes);

    int gcount = (rb_end - rb_begin < G) ? (rb_end - rb_begin) : G;
    int units = gcount * nbc * SPL;   // work items of the pass
    // Which unit the k-th work item of a pass is.  Batch >= 4: column blocks first, so that the
    // wavefronts that run side by side work on the same column block of different row blocks and
    // share its activation fragments (2 KiB per batch row and unit) in the L1.
    constexpr bool COLMAJOR = (BP >= QP_COLMAJOR_MIN_BP) && !SPLIT;
    auto unit_of = [&](int k, int gc) __attribute__((always_inline)) -> int {
        if constexpr (!COLMAJOR) return k;
        const int C = k / gc;
        return (k - C * gc) * nbc + C;
    };
    int k = wave;                                  // work item of this wavefront in the pass
    int u = (k < units) ? unit_of(k, gcount) : 0;  // its unit
    // A wavefront without an item loads item 0 as well, to keep this code free of branches;
    // it only skips the arithmetic.
    const int uw = u;
    const int uu = uw / SPL;                                        // its unit
    const bool half1 = SPLIT && __builtin_amdgcn_readfirstlane(uw & 1);   // its half of the unit
    // Activation fragments first: they hit in L2, come back early, and - loads returning in
    // issue order - let step 0 start as soon as the first piece of codes has landed.
    const int g = lane >> 4, j = lane & 15;
    const int tj = j & (TT - 1);
    const int bj = j / TT;
    const bool xlive = bj < B;  // columns beyond the batch re-read row 0; their results are dropped
    // Activations either row-major [B, ldx] (fragment n of column block C: 16 bytes per lane
    // at row bj, column 1024 C + 256 g + 8 (TT n + tj)) or already in fragment order
    // (x_packed: fragment n of column block C is the 1 KiB at ((C NXF + n) 64 + lane) 16).
    // XL: fragment order in LDS, written by the rotation below.
    // (not for the V = 1 trellis: bound by its table lookups, and with the buffer form the compiler's
    // register allocation at batch 9 - 16 came out worse for 2 and 4 bits - 19.7 -> 23.7 us, 24.7 -> 36.4 us)
    constexpr bool XBUF = !XL && BP >= 8 && S != QP_TCQ;
    // the lane's part of the address: a 32-bit byte offset (the host checks that it fits) or its pointer
    const uint32_t xlo = x_packed ? 16u * lane : 2u * ((uint32_t)(xlive ? bj : 0) * (uint32_t)ldx + 256u * g + 8u * tj);
    const half_t *xlane = XL ? xr_lds + 8 * qp_xr_swizzle_lane(lane)
                             : (x_packed ? x + 8 * lane : x + (int64_t)(xlive ? bj : 0) * ldx + 256 * g + 8 * tj);
    const int xcs = (XL || x_packed) ? 1024 * BP : 1024;   // halves between column blocks
    const int xfs = (XL || x_packed) ? 512 : 8 * TT;       // halves between fragments
    // extent of the activations in bytes: a load beyond it would return zeros instead of faulting
    const uint32_t xbytes = x_packed ? (uint32_t)nbc * (2048u * BP) : 2u * ((uint32_t)(B - 1) * (uint32_t)ldx + (uint32_t)w.N);
    // N % 1024 != 0 (N % 256 == 0: 11008, 13824 ...): the last column block has only tail_cols / 256 of its
    // four lane groups.  The codes of the others are padding (zero bytes in the native layout; in the
    // canonical one the lane re-reads group 0), their activations are fetched from group 0's address -
    // which exists - and masked to zero.
    const int tail_cols = TN ? (w.N & 1023) : 0;
    const bool g_beyond = TN && tail_cols != 0 && 256 * g >= tail_cols;
    const uint32_t x_keep = g_beyond ? 0u : 0xffffffffu;
    const int x_back = (XL || x_packed) ? 0 : 256 * g;   // halves back to group 0 (row-major activations)
    auto x_at = [&](int C) __attribute__((always_inline)) {
        const bool tail = TN && tail_cols != 0 && C == nbc - 1;
        const int back = (tail && g_beyond) ? x_back : 0;
        if constexpr (XBUF)
            return QpXBuf{__builtin_amdgcn_make_buffer_rsrc(const_cast<half_t *>(x), 0, (int)xbytes, 0x00020000),
                          2 * C * xcs, xlo - 2u * (uint32_t)back, 2 * xfs, tail, x_keep};
        else
            return QpXPtr{xlane + C * xcs - back, 0u, xfs, tail, x_keep};
    };
    const bool owner = (tj == 0) && xlive;  // lane (g, b*TT) ends up with rows 4g..4g+3 of batch row b
    // block (row block rb0 + slot, column block C) of unit u = slot * nbc + C, and whether
    // it has all P pieces
    const int hcb = nbc >> 1;   // half-TCQ: column blocks per half
    // First piece of this lane for unit un = slot * nbc + C of the pass that starts at row block rb0.
    const bool canonical = w.layout == QP_LAYOUT_CANONICAL;
    const int ps = canonical ? 1 : 64;
    auto unit_block = [&](int rb0, int un, int C, bool &full) -> const u32x4_t * {
        const int slot = (un * nbc_magic) >> 16;
        if constexpr (HH) full = __builtin_amdgcn_readfirstlane(C >= hcb);
        else full = true;
        if (canonical) {
            // row 16 (rb0 + slot) + i of the bitstream; its span for columns 1024 C + 256 g ..
            int64_t off;
            if constexpr (HH)
                off = full ? (int64_t)hcb * (64 * CB) + (int64_t)((C - hcb) * 4 + (lane >> 4)) * (16 * (CB + 1))
                           : (int64_t)(C * 4 + (lane >> 4)) * (16 * CB);
            else
                off = (int64_t)(C * 4 + ((g_beyond && C == nbc - 1) ? 0 : (lane >> 4))) * T::SPAN;
            return reinterpret_cast<const u32x4_t *>(w.codes + ((int64_t)(rb0 + slot) * 16 + (lane & 15)) * w.row_stride + off);
        }
        if constexpr (HH) {
            return codes16 + (int64_t)(rb0 + slot) * (hcb * 64 * (2 * CB + 1)) + C * (64 * CB) +
                   (full ? (C - hcb) * 64 : 0) + lane;
        } else {
            return codes16 + ((int64_t)rb0 * nbc + un) * BLK16 + lane;
        }
    };
    uint16_t scale_first = 0;
    typename D::Lane lc = D::lane_const();
    // The first pass in two instances: for a wavefront that has a work item - the straight-line code below, no
    // branch around any load, so that every wait can name exactly the loads it needs - and for one that has none
    // (the trellis kernels always run 16 wavefronts, the kernels that rotate the activations themselves 8 or 16),
    // which takes part in the table build, the transform's constants and every barrier but requests nothing.
    // (Such a wavefront used to load item 0 as well, to keep this code free of branches: on a layer of four units
    // per workgroup twelve wavefronts' worth of requests queued in front of the four that mattered.)
    auto first_pass = [&](auto act_c) __attribute__((always_inline)) {
        constexpr bool ACT = decltype(act_c)::value != 0;      // 0: no work item
        constexpr bool FETCH = decltype(act_c)::value == 1;    // 2: an item, but no chunk of the block to rotate (XL == 1)
        half8_t xf[PF];
        const auto xu = x_at(uu - ((uu * nbc_magic) >> 16) * nbc);   // column block = uu % nbc
        const int xn0 = half1 ? PF : 0;   // first fragment of this item
        // XL: the unrotated activations and their signs are requested first, ahead of the weights
        QpHad1024In rin0;
        QpHad1024 had;
        if constexpr (XL == 2) {
            // block `wave` (a wavefront without one fetches the last block instead - no branch around the
            // loads - and drops it)
            const int c0 = wave < nbc ? wave : nbc - 1;
            if constexpr (ACT) rin0 = qp_fwht1024_fetch(x + 1024 * c0, signs + 1024 * c0, lane);
        } else if constexpr (XL == 1) {
            // chunk `wave` of the one block (a wavefront beyond the last chunk fetches the last one again - no
            // branch around the loads - and drops it)
            const int nch = rot_block >> 10;
            if constexpr (FETCH) rin0 = qp_fwht1024_fetch(x + 1024 * (wave < nch ? wave : nch - 1), signs + 1024 * (wave < nch ? wave : nch - 1), lane);
        } else if constexpr (ACT) {
    #pragma unroll
            for (int n = 0; n < PF; ++n) xf[n] = xu.frag(xn0 + n);
        }
        // XL == 2: the constant matrices of the transform are worked out by the workgroup once, one dword
        // per thread, in front of a table build (whose barriers publish them) and behind the first loads:
        // vector work in front of loads delays them, four wavefronts share a SIMD.
        auto rotate_consts = [&]() __attribute__((always_inline)) {
            if constexpr (XL != 0) QpHad1024::fill(had_lds, wgt);
        };
        u32x4_t q[P];
        bool full;
        QP_T(14);
        {
            const u32x4_t *blk = unit_block(rb_begin, uu, uu - ((uu * nbc_magic) >> 16) * nbc, full);
            if constexpr (MID_BUILD) {
                // The trellis tables (64 / 128 KiB of LDS writes, two barriers) are built with the activation
                // fragments and the first piece already requested and the other pieces still to be asked
                // for: every wavefront reaches the barriers without waiting in the load queue, and the
                // first data arrives while the table is written (5 - 7 % on 4096x4096 and 28672x4096).
                if constexpr (!ACT) {
                } else if constexpr (SPLIT) {
                    if (half1) qp_half_pieces_load<S, CB, P, 1, 1>(blk, ps, q);
                    else qp_half_pieces_load<S, CB, P, 0, 1>(blk, ps, q);
                } else {
                    q[0] = qp_stream_load(blk);
                }
                rotate_consts();
                D::build(tab, reinterpret_cast<uint16_t *>(red), pre, wgt);
                if constexpr (!ACT) {
                } else if constexpr (SPLIT) {
                    if (half1) qp_half_pieces_load<S, CB, P, 1, 2>(blk, ps, q);
                    else qp_half_pieces_load<S, CB, P, 0, 2>(blk, ps, q);
                } else {
    #pragma unroll
                    for (int p = 1; p < P; ++p) {
                        if (HH && p == P - 1) {   // half-TCQ: the last piece only exists in the second half
                            q[p] = u32x4_t{0u, 0u, 0u, 0u};
                            if (full) q[p] = qp_stream_load(blk + p * ps);
                        } else {
                            q[p] = qp_stream_load(blk + p * ps);
                        }
                    }
                }
            } else if constexpr (SPLIT) {
                if constexpr (ACT) {
                    if (half1) qp_half_pieces_load<S, CB, P, 1>(blk, ps, q);
                    else qp_half_pieces_load<S, CB, P, 0>(blk, ps, q);
                }
                rotate_consts();
            } else {
                if constexpr (MOVABLE && !HH) {
                    // A table shared by the workgroup that is built "before the loads" is built with the
                    // activation fragments and the first piece(s) already on their way: the fetch of its
                    // source, 32 - 64 KiB of LDS writes and a barrier take most of a microsecond, the few
                    // early requests are accepted without back-pressure, and - loads returning in order -
                    // step 0 can start as soon as the table stands.
                    // (measured with one, two and three pieces ahead of the build: one is best)
                    if constexpr (ACT) q[0] = qp_stream_load(blk);
                    rotate_consts();
                    if (!table_late) D::build(tab, reinterpret_cast<uint16_t *>(red), pre, wgt);
                    if constexpr (ACT) {
    #pragma unroll
                        for (int p = 1; p < P; ++p) q[p] = qp_stream_load(blk + p * ps);
                    }
                } else {
                    if constexpr (ACT) qp_pieces_load<P, HH>(blk, ps, full, q);
                    rotate_consts();
                }
            }
        }
        // the first output this thread stores after the pass: its per-row scale is fetched now
        {
            const int o = threadIdx.x;
            const int i = o & 15, slot = o >> (4 + LB);
            scale_first = w.scales[(slot < gcount) ? (rb_begin + slot) * 16 + i : 0];
        }
        QP_T(7);
        // XL == 1: the first W = rot_block / 1024 wavefronts transform a chunk of 1024 each on the matrix cores
        // and park it in LDS; 256 threads then run the stages across the chunks and write the rotated block in
        // fragment order (same code as the stand-alone kernel, so the same bits).  Where the parking room borrows
        // the table's, the table is built afterwards; otherwise before, while the activations are on their way.
        auto rotate_chunks = [&]() __attribute__((always_inline)) {
            if constexpr (XL == 1) {
                __syncthreads();              // the constant matrices stand
                QP_T(18);
                if (wave < (rot_block >> 10)) {
                    had.read(had_lds, lane);
                    float4_t o[2][2];
                    qp_fwht1024_run(had, rin0, o);
                    qp_fwht_park(rot_buf + 1024, wave, lane, o);   // behind the constant matrices
                }
            }
        };
        auto rotate_across = [&]() __attribute__((always_inline)) {
            if constexpr (XL == 1) {
                const float *ex = rot_buf + 1024;
                const int nch = rot_block >> 10;
                __syncthreads();
                if (threadIdx.x < 256) {
                    auto put = [&](int idx, uint2 v) { *reinterpret_cast<uint2 *>(xr_lds + qp_xr_swizzled(qp_xr_index(0, idx, 0, 1))) = v; };
                    const float scale = rot_norm * 32.0f;
                    if (nch == 1) qp_fwht_cross<1>(threadIdx.x, ex, scale, put);
                    else if (nch == 2) qp_fwht_cross<2>(threadIdx.x, ex, scale, put);
                    else if (nch == 4) qp_fwht_cross<4>(threadIdx.x, ex, scale, put);
                    else qp_fwht_cross<8>(threadIdx.x, ex, scale, put);
                }
                QP_T(19);
                __syncthreads();
                if constexpr (ACT) {
    #pragma unroll
                    for (int n = 0; n < PF; ++n) xf[n] = xu.frag(xn0 + n);
                }
            }
        };
        // (Measured slower with the late table build between the two halves: 4096x4096 at 2.5 bits 4.9 -> 5.3 us.)
        if constexpr (!MID_BUILD) {
            if (!MOVABLE || table_late) D::build(tab, reinterpret_cast<uint16_t *>(red), pre, wgt);
        }
        rotate_chunks();
        rotate_across();
        if constexpr (XL == 2) {
            // Every wavefront transforms the block of its own unit on the matrix cores while its weights are
            // on their way, and writes it to LDS in fragment order (four consecutive elements = 8 bytes).
            // The workgroup has one row block and a wavefront per column block (the host checks), so a
            // wavefront only ever reads what it wrote itself - LDS operations of a wavefront complete in
            // order - and nobody waits for anybody.
            if constexpr (!QpLinLds<D, S, CB, BP>::TABLE_HAS_BARRIER) __syncthreads();   // the constant matrices
            had.read(had_lds, lane);
            QP_T(18);
            // (Transforming in front of an early table build instead - the SIMDs are idle there - delays the
            // remaining loads by as much as it saves: 8.3 against 8.1 us on 4096x14336 at 2.5 bits.)
            if (wave < nbc) {
                float4_t o[2][2];
                qp_fwht1024_run(had, rin0, o);
    #pragma unroll
                for (int tb = 0; tb < 2; ++tb)
    #pragma unroll
                    for (int ta = 0; ta < 2; ++ta)
                        *reinterpret_cast<uint2 *>(xr_lds + qp_xr_swizzled(qp_xr_index(0, 1024 * wave + qp_fwht1024_elem(lane, tb, ta), 0, 1))) =
                            qp_fwht1024_pack(o[tb][ta]);
            }
            QP_T(19);
            // (two wavefronts per unit: a wavefront's half units belong to other column blocks than the one
            // it transformed, so here everybody does wait for everybody)
            if constexpr (SPLIT) __syncthreads();
            if constexpr (ACT) {
    #pragma unroll
                for (int n = 0; n < PF; ++n) xf[n] = xu.frag(xn0 + n);
            }
        }
        QP_T(1);
        if (ACT && k < units) {
            float4_t v;
            if constexpr (SPLIT) {
                if (half1) v = qp_unit_compute<D, P, PF, TT, 16, 32>(q, xf, xu, tab, lc, pre);
                else v = qp_unit_compute<D, P, PF, TT, 0, 16>(q, xf, xu, tab, lc, pre);
            } else if constexpr (HH) {
                if (full) v = qp_unit_compute<D, P, PF, TT>(q, xf, xu, tab, lc, pre);
                else v = qp_unit_compute<typename D::Lo, P, PF, TT>(q, xf, xu, tab, lc, pre);
            } else {
                v = qp_unit_compute<D, P, PF, TT>(q, xf, xu, tab, lc, pre);
            }
            if (owner) *reinterpret_cast<float4_t *>(&red[(u * BP + bj) * 16 + 4 * g]) = v;
        }
    };
    // (the scalar and vector quantizers without a rotation of their own run as many wavefronts as a pass has units,
    // at least four: the few that can be left over there keep the old way)
    constexpr bool IDLE_INSTANCE = XL != 0 || S == QP_TCQ || S == QP_TCQH || S == QP_TCQHH;
    if (!IDLE_INSTANCE || k < units) {
        if (XL == 1 && wave >= (rot_block >> 10)) first_pass(std::integral_constant<int, 2>{});   // (see FETCH)
        else first_pass(std::integral_constant<int, 1>{});
    } else {
        first_pass(std::integral_constant<int, 0>{});
    }
    QP_T(2);
    int rb0 = rb_begin;
    k += nw;
#ifdef QP_TRACE
    uint64_t tr_wait = 0, tr_dec = 0, tr_units = 0;
#endif
    // A workgroup whose only pass has no more work items than wavefronts (XL == 2: always, the host checks): nothing
    // follows the first pass but its sums.  Spelled out because the compiler otherwise sets up the loops below - some
    // fifty instructions of addresses and constants - between a wavefront's last multiply and the barrier that the
    // whole workgroup waits at (one-launch steps of 4096x14336: 2.5 bits 7.39 -> 7.21 us, hybrid trellis at 2 bits
    // 8.20 -> 7.94, 3.5 bits 8.53 -> 8.27, 4-bit scalar 8.39 -> 8.16 us).
    constexpr bool ONE_PASS = (XL == 2) && !SPLIT;
    const bool one_pass = ONE_PASS || (units <= nw && rb_begin + G >= rb_end);   // the same for every wavefront
    if (one_pass) qp_pass_store<BP>(w, red, y, ldy, B, rb0, gcount, nbc * SPL, scale_first, wgt);
    else while (true) {
        // ---- remaining units of this pass ----------------------------------------------
        for (; k < units; k += nw) {
            u = unit_of(k, gcount);
            const int ub = u / SPL;
            const bool h2 = SPLIT && __builtin_amdgcn_readfirstlane(u & 1);
            const int C = ub - ((ub * nbc_magic) >> 16) * nbc;
            const auto xu2 = x_at(C);
            u32x4_t q2[P];
            half8_t xf2[PF];
            bool full2;
            const u32x4_t *blk2 = unit_block(rb0, ub, C, full2);
            float4_t v;
            if constexpr (SPLIT) {
                const int n0 = h2 ? PF : 0;
#pragma unroll
                for (int n = 0; n < PF; ++n) xf2[n] = xu2.frag(n0 + n);
                if (h2) {
                    qp_half_pieces_load<S, CB, P, 1>(blk2, ps, q2);
                    v = qp_unit_compute<D, P, PF, TT, 16, 32>(q2, xf2, xu2, tab, lc, pre);
                } else {
                    qp_half_pieces_load<S, CB, P, 0>(blk2, ps, q2);
                    v = qp_unit_compute<D, P, PF, TT, 0, 16>(q2, xf2, xu2, tab, lc, pre);
                }
                if (owner) *reinterpret_cast<float4_t *>(&red[(u * BP + bj) * 16 + 4 * g]) = v;
                continue;
            }
            qp_unit_load<P, PF, HH>(blk2, ps, xu2, full2, q2, xf2);
            QP_T(8);
#ifdef QP_TRACE
            const uint64_t tr_a = __builtin_amdgcn_s_memtime();
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            const uint64_t tr_b = __builtin_amdgcn_s_memtime();
#endif
            if constexpr (HH) {
                if (full2) v = qp_unit_compute<D, P, PF, TT>(q2, xf2, xu2, tab, lc, pre);
                else v = qp_unit_compute<typename D::Lo, P, PF, TT>(q2, xf2, xu2, tab, lc, pre);
            } else {
                v = qp_unit_compute<D, P, PF, TT>(q2, xf2, xu2, tab, lc, pre);
            }
            if (owner) *reinterpret_cast<float4_t *>(&red[(u * BP + bj) * 16 + 4 * g]) = v;
            QP_T(9);
#ifdef QP_TRACE
            tr_wait += tr_b - tr_a;
            tr_dec += __builtin_amdgcn_s_memtime() - tr_b;
            tr_units += 1;
#endif
        }
        qp_pass_store<BP>(w, red, y, ldy, B, rb0, gcount, nbc * SPL, scale_first, wgt);
        // ---- next pass ------------------------------------------------------------------
        rb0 += G;
        if (rb0 >= rb_end) break;
        gcount = (rb_end - rb0 < G) ? (rb_end - rb0) : G;
        units = gcount * nbc * SPL;
        k = wave;
        {
            const int o = threadIdx.x;
            const int i = o & 15, slot = o >> (4 + LB);
            scale_first = w.scales[(slot < gcount) ? (rb0 + slot) * 16 + i : 0];
        }
    }
    QP_T(6);
    QP_T(17);
#ifdef QP_TRACE
    if ((threadIdx.x & 63) == 0 && tr_units) {
        uint64_t *tb = &qp_trace_lds[(threadIdx.x >> 6) * QP_TS];
        tb[10] = tr_wait; tb[11] = tr_dec; tb[12] = tr_units;
    }
    QP_T_FLUSH();
#endif
}


// XL (batch 1 only): the workgroup rotates the activations itself; a kernel of its own, so that the
// plain kernel does not carry the transform's LDS arrays and more workgroups fit a compute unit.
template <int S, int CB, int BP, bool SPLIT, int XL, bool TN = false>
__global__ __launch_bounds__(1024) void k_linear_mfma(QpW w, const half_t *x, int B, int64_t ldx, half_t *y,
                                                      int64_t ldy, int G, int rb_q, int rb_r, int nbc_magic,
                                                      int x_packed, const int8_t *signs, int rot_block, float rot_norm) {
    using D = typename QpDecSel<S, CB, SPLIT, BP>::type;
    using L = QpLinLds<D, S, CB, BP>;
    // The 2.5-bit vector quantizer with its table of code pairs and no rotation of its own requests every kernel
    // argument here, in one go.  Left to itself the compiler fetches each where it is first used, and the three
    // cache lines of the argument block are then missed one after the other, each with a wait of its own, in
    // front of the first loads of a wavefront (layer alone: 4096x14336 6.62 -> 6.53 us, batch 2 7.02 -> 6.95,
    // batch 16 12.43 -> 12.29, 4096x4096 3.75 -> 3.67 us, 8192x8192 6.84 -> 6.76 us).  Not the others: 4-bit scalar
    // and 3.5-bit pairs measured the same or a per cent slower, and where the first request - the table's source
    // - only needs the first line, waiting for all three delays it (hybrid trellis 4096x14336 at 2 bits
    // 7.83 -> 8.02 us, 4096x4096 at 4 bits 5.17 -> 5.29 us; the one-launch step at 2.5 bits 7.46 -> 7.51 us).
    if constexpr (XL == 0 && S == QP_VQ && CB == 5 && BP != 4) {
        asm volatile("" ::"s"(w.codes), "s"(w.lut), "s"(w.scales), "s"(w.M), "s"(w.N), "s"(w.row_stride), "s"(w.layout),
                     "s"(w.nbc), "s"(x), "s"(B), "s"(ldx), "s"(y), "s"(ldy), "s"(G), "s"(rb_q), "s"(rb_r), "s"(nbc_magic),
                     "s"(x_packed), "s"(blockDim.x));
    }
    static_assert(XL == 0 || L::ROT, "in-kernel rotation: batch 1");
    static_assert(XL != 2 || L::ROTM, "per-wavefront rotation: tables of at most 64 KiB");
    // One object, the table first: at LDS address 0 a lookup's address register is the whole address;
    // anywhere above 64 KiB (where the compiler would put it once another array grows larger than it)
    // every lookup costs a vector add for the base.
    struct Lds {
        __attribute__((aligned(16))) uint8_t tab[D::TAB_BYTES];
        // [unit][b][row]; before the first pass the same room stages a table's source
        __attribute__((aligned(16))) float red[L::RED];
        __attribute__((aligned(16))) half_t xr[XL == 2 ? L::ROTM_MAX : XL == 1 ? L::ROT_MAX : 0];   // (empty without in-kernel rotation)
        __attribute__((aligned(16))) float rot[XL == 2 ? 1024 : XL == 1 ? L::ROT_SCRATCH_FLOATS : 0];
    };
    __shared__ Lds lds;
    if constexpr (XL == 2) {
        qp_linear_body<S, CB, BP, 2, SPLIT>(w, x, B, ldx, y, ldy, G, rb_q, rb_r, nbc_magic, x_packed, signs,
                                            rot_block, rot_norm, lds.tab, lds.red, lds.xr, lds.rot);
    } else if constexpr (XL == 1) {
        qp_linear_body<S, CB, BP, 1, SPLIT>(w, x, B, ldx, y, ldy, G, rb_q, rb_r, nbc_magic, x_packed, signs,
                                            rot_block, rot_norm, lds.tab, lds.red, lds.xr, lds.rot);
    } else {
        qp_linear_body<S, CB, BP, 0, SPLIT, TN>(w, x, B, ldx, y, ldy, G, rb_q, rb_r, nbc_magic, x_packed, signs,
                                                rot_block, rot_norm, lds.tab, lds.red, nullptr, nullptr);
    }
}

// Half units exist for the trellis schemes at batch <= 2 (the kernels that are bound by their
// own decode work when a workgroup has few units).
template <int S, int CB, int BP, bool SPLIT>
static void qp_launch_xl(int grid, int nw, hipStream_t st, const QpW &w, const void *x, int B, int64_t ldx, void *y,
                         int64_t ldy, int G, int rb_q, int rb_r, int nbc_magic, int x_packed, const int8_t *signs,
                         int rot_block, float rot_norm) {
    if constexpr (BP == 1) {
        using D = typename QpDecSel<S, CB, SPLIT, BP>::type;
        if constexpr (QpLinLds<D, S, CB, BP>::ROTM) {
            if (rot_block > 0 && rot_block != w.N) {
                hipLaunchKernelGGL((k_linear_mfma<S, CB, BP, SPLIT, 2>), dim3(grid), dim3(64 * nw), 0, st, w,
                                   (const half_t *)x, B, ldx, (half_t *)y, ldy, G, rb_q, rb_r, nbc_magic, x_packed,
                                   signs, rot_block, rot_norm);
                return;
            }
        }
        if constexpr (QpLinLds<D, S, CB, BP>::ROT) {
            if (rot_block > 0) {
                hipLaunchKernelGGL((k_linear_mfma<S, CB, BP, SPLIT, 1>), dim3(grid), dim3(64 * nw), 0, st, w,
                                   (const half_t *)x, B, ldx, (half_t *)y, ldy, G, rb_q, rb_r, nbc_magic, x_packed,
                                   signs, rot_block, rot_norm);
                return;
            }
        }
    }
    if constexpr (!SPLIT) {
        if (w.N % 1024 != 0) {   // the last column block is cut short
            hipLaunchKernelGGL((k_linear_mfma<S, CB, BP, false, 0, true>), dim3(grid), dim3(64 * nw), 0, st, w,
                               (const half_t *)x, B, ldx, (half_t *)y, ldy, G, rb_q, rb_r, nbc_magic, x_packed, signs,
                               rot_block, rot_norm);
            return;
        }
    }
    hipLaunchKernelGGL((k_linear_mfma<S, CB, BP, SPLIT, 0>), dim3(grid), dim3(64 * nw), 0, st, w,
                       (const half_t *)x, B, ldx, (half_t *)y, ldy, G, rb_q, rb_r, nbc_magic, x_packed, signs,
                       rot_block, rot_norm);
}

template <int S, int CB, int BP>
static void qp_launch_one(bool split, int grid, int nw, hipStream_t st, const QpW &w, const void *x, int B,
                          int64_t ldx, void *y, int64_t ldy, int G, int rb_q, int rb_r, int nbc_magic, int x_packed,
                          const int8_t *signs, int rot_block, float rot_norm) {
    constexpr bool CAN_SPLIT = (qp_alt_splits(S) && BP <= 2) || (S == QP_VQ && CB == 5 && BP <= 4);
    if constexpr (CAN_SPLIT) {
        if (split) {
            qp_launch_xl<S, CB, BP, true>(grid, nw, st, w, x, B, ldx, y, ldy, G, rb_q, rb_r, nbc_magic, x_packed,
                                          signs, rot_block, rot_norm);
            return;
        }
    }
    qp_launch_xl<S, CB, BP, false>(grid, nw, st, w, x, B, ldx, y, ldy, G, rb_q, rb_r, nbc_magic, x_packed, signs,
                                   rot_block, rot_norm);
}

// Whether the block kernel can rotate N / 1024 blocks of 1024 itself at batch 1: every workgroup has
// one row block (M <= 4096) and a wavefront per column block (N <= 16384), and the rotated row fits
// into LDS beside the table (not beside the 128 KiB one of the V = 1 trellis).  Larger layers take
// the two launches: with several units per wavefront the transform would need a workgroup barrier
// behind it, and measured no faster (8192 x 28672: 22.6 against 22.3 us).
bool qp_linear_rotates_blocks(int scheme, int M, int N, int rot_block) {
    return rot_block == 1024 && N > 1024 && N % 1024 == 0 && N <= 16384 && M <= 4096 && scheme != QP_TCQ;
}

qp_status qp_launch_linear_mfma(const QpW &w, int scheme, int cb, const void *x, int B, int64_t ldx, void *y,
                                int64_t ldy, int x_packed, const int8_t *signs, int rot_block, hipStream_t st) {
    const int nbc = w.nbc, rbk = w.M / 16;
    if (nbc < 1 || nbc > QP_NBC_MAX) return QP_ERR_UNSUPPORTED;
    int umax = qp_umax(B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : B <= 8 ? 8 : 16, scheme == QP_TCQ);
    // Batch 5 - 16: passes of 64 units only where 32 would hold a single row block (more than 16 column
    // blocks): two row blocks per pass let pairs of wavefronts share a column block's activation fragments
    // in the L1 (8192x28672 at 3.5 bits, batch 8: 31.2 -> 29.1 us per step); with four row blocks in 32
    // units already, 64 measured the same or slower.
    if (B > 4 && nbc <= 16 && umax > 32) umax = 32;
    // Tuning options: workgroups per compute unit and wavefronts per workgroup.
    int wg_per_cu = qp_opt(QP_OPT_WG_PER_CU), nw_forced = qp_opt(QP_OPT_NW);
    const bool big_table = (scheme == QP_TCQ || scheme == QP_TCQH || scheme == QP_TCQHH);
    if (big_table) { wg_per_cu = 1; nw_forced = 0; }
    int grid = rbk < 256 * wg_per_cu ? rbk : 256 * wg_per_cu;
    int rb_per_wg = (rbk + grid - 1) / grid;
    int G = umax / nbc;
    if (G > rb_per_wg) G = rb_per_wg;
    int units = G * nbc;
    int rb_q = rbk / grid, rb_r = rbk % grid;
    int nbc_magic = (65536 + nbc - 1) / nbc;  // u / nbc == (u * magic) >> 16 for u < 1024
    // Two wavefronts per unit (trellis schemes, batch <= 2, a pass with no more units than the workgroup
    // has wavefronts) spread the decode work over all SIMDs, but the pieces both halves need are read
    // twice and twice as many wavefronts queue for the load path.  Measured per call, one / two wavefronts
    // per unit: 4096x14336 at 3 bits V = 1 15.8 / 16.2 us, hybrid at 2, 4 and 5 bits 8.1 / 8.3, 9.4 / 10.2
    // and 11.1 / 12.0 us, 4096x8192 at 3 bits hybrid 6.7 / 6.9 us; only 4096x4096 at 3 bits hybrid
    // gains (5.4 / 5.2 us).  So: off unless QP_OPT_LINEAR_SPLIT = 1 asks for it where it is legal.
    const int split_opt = qp_opt(QP_OPT_LINEAR_SPLIT);
    const bool can_split = (scheme == QP_TCQ || scheme == QP_TCQH) && B <= 2 && units <= 16 && w.N % 1024 == 0;
    bool split = false;
    if (split_opt == 0) split = false;
    if (split_opt == 1) split = can_split;
    // VQ 5 bit: the per-wavefront table (32 entries, one code per lookup, no workgroup barrier in front of the
    // decode) where it measured faster than the workgroup's table of code pairs: batch 3 - 4 with 9 to 16
    // units per workgroup (us per call, per-wavefront / shared: 4096x14336 batch 4 7.9 / 8.6, 4096x12288
    // 6.9 / 7.5; the same at batch 3 and from 8 units down; at batch 9 - 16 with fragment-order activations
    // the shared table wins since it holds pairs, 4096x14336 12.75 / 12.6, 4096x8192 8.8 / 8.6).
    const int units_wg = rb_per_wg * nbc;
    if (scheme == QP_VQ && cb == 5 && units_wg <= 16 && B > 2 && B <= 4 && units_wg > 8) {
        split = split_opt != 0;
    }
    // VQ 5 bit at batch 1 - 2: the sixteen-copy table of code pairs (128 KiB, no lookup collisions) where its
    // longer build is paid back on every machine it was measured on - from 20 units per workgroup on, and at
    // 7 - 8 units, where the table is built behind the loads anyway; never with the rotation inside the kernel,
    // which has no room beside it.  Two kinds of machine turned up, told apart by the one-launch step of
    // 4096x14336 (7.3 us on one, 8.1 us on the other: whatever runs on the SIMDs and the LDS in front of the
    // decode - table build, transform - takes longer there).  us per call at batch 1, eight / sixteen copies, by
    // units per workgroup, on the first kind: 4 (4096x4096) 3.77 / 3.88, 5 4.33 / 4.42, 6 4.48 / 4.48, 7
    // 4.64 / 4.61, 8 (4096x8192, 2048x8192) 4.87 / 4.78, 4.62 / 4.45, 9 5.55 / 5.84, 10 5.69 / 5.90, 12
    // 6.07 / 6.04, 13 6.58 / 6.50, 14 (4096x14336) 6.66 / 6.50, 16 (4096x16384, 8192x8192) 7.03 / 6.78,
    // 6.85 / 6.63, 20 (10240x8192) 8.34 / 8.01, 28 (8192x14336) 11.09 / 10.82, 49 (14336x14336) 16.73 / 16.20;
    // on the second kind: 8 4.96 / 4.85, 4.60 / 4.41, 14 6.77 / 6.89, 16 7.25 / 7.66, 7.09 / 7.49, 20 9.11 / 8.78,
    // 28 11.36 / 10.98, 49 17.63 / 16.92.  Batch 2 follows batch 1 (14 units: 7.03 / 6.67 and 7.27 / 7.45).
    if (scheme == QP_VQ && cb == 5 && B <= 2) {
        const bool pays = units_wg >= 20 || units_wg == 7 || units_wg == 8;
        split = (split_opt < 0 ? pays : split_opt == 1) && rot_block <= 0;
    }
    if (w.N % 1024 != 0) split = false;   // a last column block cut short: the plain form only
    int nw = units < 16 ? units : 16;
    if (scheme == QP_TCQ || scheme == QP_TCQH || scheme == QP_TCQHH) nw = 16;  // the table staging is written for 1024 threads
    if (nw_forced >= 4 && nw_forced <= 16 && nw_forced < nw) nw = nw_forced;
    if (nw < 4) nw = 4;
    const float rot_norm = rot_block > 0 ? 1.0f / sqrtf((float)rot_block) : 0.f;
    if (rot_block > 0) {
        if (B != 1) return QP_ERR_UNSUPPORTED;
        if (rot_block == w.N) {
            // in-kernel rotation of one block; up to 8 wavefronts transform it
            if (rot_block > 8192 || rot_block < 1024 || scheme == QP_TCQ) return QP_ERR_UNSUPPORTED;
            if (nw < 8) nw = 8;
        } else {
            // N / 1024 blocks of 1024, one per wavefront
            if (!qp_linear_rotates_blocks(scheme, w.M, w.N, rot_block) || rb_per_wg != 1) return QP_ERR_UNSUPPORTED;
            nw = 16;
        }
    }
    // A table that the whole workgroup shares is built after the first loads have been issued when
    // the workgroup has few units, and at batch >= 4 with row-major activations (whose many
    // small loads then start earlier); before them otherwise.
    // (few units = what they request fits the compute unit's window of loads in flight, so nobody
    // queues in front of the build's barriers: at most 56 KiB of codes, and at most 8 units.
    // 4 bit scalar at batch 1, 8 units of 8 KiB: 5.9 us late, 5.6 us early.)
    const int unit_kib = (scheme == QP_SQ) ? 2 * cb : cb;   // of the schemes with such a table: 4 bit scalar, 5 and 7 bit pairs
    int late_few = 56 / (unit_kib > 0 ? unit_kib : 1);
    if (late_few > 8) late_few = 8;
    int late_max = (!x_packed && B >= 4) ? 1024 : late_few;
    if (const int forced = qp_opt(QP_OPT_TABLE_LATE_MAX); forced >= 0) late_max = forced;
    const int x_flags = (x_packed ? 1 : 0) | (late_max << 8);
#define CALL_BP(S, C, BP) \
    qp_launch_one<S, C, BP>(split, grid, nw, st, w, x, B, ldx, y, ldy, G, rb_q, rb_r, nbc_magic, x_flags, signs, \
                            rot_block, rot_norm)
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

// ------------------------------------------------------------------ dequantize only, native layout
// Same units, piece loads and table lookups as the fused kernel, without the multiply
// (Appendix D, dequantization-only kernels).  Write-bound: 2 bytes out per weight.  After
// step s lane (i, g) holds the 8 weights of row i, columns 256 g + 8 s .. + 7 of its block;
// storing that directly would scatter 16-byte pieces over 64 cache lines per instruction
// (measured 2.5 TB/s).  Four steps at a time therefore go through a 4 KiB LDS tile per
// wavefront (swizzled, conflict-free both ways) so that four neighbouring lanes store the
// 64 contiguous bytes one lane decoded.  Blocks are dealt round-robin to the decoding
// wavefronts of the grid; with the 128 KiB trellis tables only 8 of the 16 wavefronts decode
// (the tiles of 16 would not fit), the others only help staging the table.
template <int S, int CB>
__global__ __launch_bounds__(1024) void k_dequant_blocks(QpW w, uint16_t *out, int nblocks) {
    using T = QpTraits<S, CB>;
    using D = QpDec<S, CB>;
    constexpr bool HH = (S == QP_TCQHH);
    constexpr int P = HH ? T::PIECES + 1 : T::PIECES;
    constexpr int BLK16 = T::BLOCK_BYTES / 16;
    constexpr int STAGE_FLOATS = T::HYBRID ? (1 << T::TLUT_BITS) : 512;
    constexpr int NWD = (D::TAB_BYTES > 65536) ? 8 : 16;   // decoding wavefronts per workgroup
    __shared__ __attribute__((aligned(16))) uint8_t tab[D::TAB_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t tile[NWD * 4096];   // also stages a table's source
    static_assert(NWD * 4096 >= STAGE_FLOATS * 4, "staging room");
    D::early(tab, reinterpret_cast<uint16_t *>(tile), w.lut);
    const typename D::Pre pre = D::pre(w.lut);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nbc = w.nbc, hcb = nbc >> 1;
    const u32x4_t *codes16 = reinterpret_cast<const u32x4_t *>(w.codes);
    typename D::Lane lc = D::lane_const();
    const int nwd = (int)(blockDim.x >> 6) < NWD ? (int)(blockDim.x >> 6) : NWD;
    const int stride = gridDim.x * nwd;
    int t = (wave < nwd) ? blockIdx.x * nwd + wave : nblocks;   // a wavefront that does not decode has no block

    u32x4_t q[P];
    bool full = true;
    auto issue = [&](int blk) __attribute__((always_inline)) {
        const bool live = blk < nblocks;
        const int bc = live ? blk : 0;
        const int R = bc / nbc, C = bc - R * nbc;
        const u32x4_t *src;
        if constexpr (HH) {
            full = __builtin_amdgcn_readfirstlane(C >= hcb);
            src = codes16 + (int64_t)R * (hcb * 64 * (2 * CB + 1)) + C * (64 * CB) + (full ? (C - hcb) * 64 : 0);
        } else {
            src = codes16 + (int64_t)bc * BLK16;
        }
        qp_pieces_load<P, HH>(src + lane, 64, full, q);
    };
    issue(t);
    if (!QpTableMovable<D>::value) D::build(tab, reinterpret_cast<uint16_t *>(tile), pre);
    __syncthreads();   // the staging room becomes the transposition tiles
    // tile of this wavefront: 64 slots of 64 bytes, slot = decoding lane, chunk c of a slot
    // at ((c + slot / 2) % 4) * 16 so that eight neighbouring lanes always cover all banks
    u32x4_t *tl = reinterpret_cast<u32x4_t *>(tile + (wave < nwd ? wave : 0) * 4096);
    const int wr = lane * 4;                            // in 16-byte units
    const int rd_slot0 = lane >> 2, rd_c = lane & 3;    // store k reads slot 16 k + lane / 4, chunk lane % 4
    while (t < nblocks) {
        const int R = t / nbc, C = t - R * nbc;
        // lane stores: row rd_slot0 of the block, column group k, chunk rd_c of every four steps
        uint16_t *dst = out + (int64_t)(R * 16 + rd_slot0) * w.N + C * 1024 + rd_c * 8;
        const bool hi = full;
        qp_static_for<0, 8>([&](auto s4c) __attribute__((always_inline)) {
            constexpr int s4 = decltype(s4c)::value;
            qp_static_for<0, 4>([&](auto cc) __attribute__((always_inline)) {
                constexpr int c = decltype(cc)::value;
                half8_t a;
                if constexpr (HH) {
                    if (hi) a = qp_step<D, P, 4 * s4 + c>(q, tab, lc, pre);
                    else a = qp_step<typename D::Lo, P, 4 * s4 + c>(q, tab, lc, pre);
                } else {
                    a = qp_step<D, P, 4 * s4 + c>(q, tab, lc, pre);
                }
                tl[wr + ((c + (lane >> 1)) & 3)] = __builtin_bit_cast(u32x4_t, a);
            });
            __builtin_amdgcn_wave_barrier();   // LDS operations of a wavefront complete in order
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int slot = 16 * k + rd_slot0;
                const u32x4_t v = tl[slot * 4 + ((rd_c + (slot >> 1)) & 3)];
                // (column group k of a last block that N cuts short is padding)
                if (C * 1024 + k * 256 < w.N) *reinterpret_cast<u32x4_t *>(dst + k * 256 + s4 * 32) = v;
            }
            __builtin_amdgcn_wave_barrier();
        });
        t += stride;
        if (t < nblocks) issue(t);
    }
}

qp_status qp_launch_dequant_blocks(const QpW &w, int scheme, int cb, void *out, hipStream_t st) {
    const int64_t nb64 = (int64_t)(w.M / 16) * w.nbc;
    if (nb64 > 0x7fffffff) return QP_ERR_SHAPE;
    const int nblocks = (int)nb64;
    const bool big_table = (scheme == QP_TCQ || scheme == QP_TCQH || scheme == QP_TCQHH);
    // small layers: fewer wavefronts per workgroup so that every CU gets some
    int nw = 16;
    if (!big_table) {
        nw = (nblocks + 255) / 256;
        if (nw < 4) nw = 4;   // the per-scheme table set-up assumes at least four wavefronts
        if (nw > 16) nw = 16;
    }
    const int nwd = (scheme == QP_TCQ) ? 8 : nw;   // decoding wavefronts: see NWD in the kernel
    int grid = (nblocks + nwd - 1) / nwd;
    if (grid > 256) grid = 256;
#define CALL(S, C) \
    hipLaunchKernelGGL((k_dequant_blocks<S, C>), dim3(grid), dim3(64 * nw), 0, st, w, (uint16_t *)out, nblocks)
    QP_DISPATCH_SCHEME(scheme, cb, CALL);
#undef CALL
    return qp_check_launch();
}
