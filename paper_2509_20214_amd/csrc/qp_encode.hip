// Quantization (the encoders): from target weights to packed codes in the canonical layout.
//   SQ / VQ : nearest table entry per weight / per pair (App. C.1, C.2 "Quantization").
//   trellis : the bitstream of a tile whose decode is closest to the 256 targets, found with the
//             Viterbi algorithm over the 2^16 states (App. C.3.1 "Quantization"), tail-biting
//             handled in two passes: an open pass over the tile rotated by half its length fixes
//             the 16 - s bits that the two ends of the stream share, a second pass constrained
//             to those bits gives the stream.
// The targets are fp16 (already rotated and scaled by the caller); distances are fp32.
#include "qp_internal.h"

typedef _Float16 half2v __attribute__((ext_vector_type(2)));

struct QpEnc {
    const half_t *W;      // targets [M, ldw]
    int64_t ldw;
    int M;
    int col0, ncols;      // column range encoded by this launch (half-TCQ: one half)
    const uint16_t *lut;  // SQ, VQ, TCQ: the table; TCQH: the small table
    uint8_t *codes;       // canonical output
    int64_t row_stride;
    int64_t code_off;     // byte offset of this range's stream inside a row
    uint8_t *back;        // trellis: gridDim.x * steps * groups bytes of decisions
    float *tile_err;      // optional, [M, tiles_row_total]
    int tiles_row_total;  // N / 256
};

// ------------------------------------------------------------------ nearest entry
// One thread: 8 consecutive weights -> one dword of 4-bit codes.  Ties go to the lower index.
__global__ __launch_bounds__(256) void k_encode_sq4(QpEnc a) {
    __shared__ float lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = qp_half_bits_to_float(a.lut[threadIdx.x]);
    __syncthreads();
    const int gpr = a.ncols >> 3;
    const int64_t total = (int64_t)a.M * gpr;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int row = (int)(t / gpr), grp = (int)(t - (int64_t)row * gpr);
        const half8_t w = *reinterpret_cast<const half8_t *>(a.W + (int64_t)row * a.ldw + a.col0 + grp * 8);
        uint32_t out = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = (float)w[e];
            int best = 0;
            float bd = fabsf(v - lut[0]);
#pragma unroll
            for (int c = 1; c < 16; ++c) {
                const float d = fabsf(v - lut[c]);
                if (d < bd) { bd = d; best = c; }
            }
            out |= (uint32_t)best << (4 * e);
        }
        *reinterpret_cast<uint32_t *>(a.codes + (int64_t)row * a.row_stride + a.code_off + grp * 4) = out;
    }
}

// One thread: 16 consecutive weights = 8 pairs -> CB bytes.
template <int CB>
__global__ __launch_bounds__(256) void k_encode_vq(QpEnc a) {
    __shared__ float lx[1 << CB], ly[1 << CB];
    for (int i = threadIdx.x; i < (1 << CB); i += blockDim.x) {
        lx[i] = qp_half_bits_to_float(a.lut[2 * i]);
        ly[i] = qp_half_bits_to_float(a.lut[2 * i + 1]);
    }
    __syncthreads();
    const int gpr = a.ncols >> 4;
    const int64_t total = (int64_t)a.M * gpr;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int row = (int)(t / gpr), grp = (int)(t - (int64_t)row * gpr);
        const half_t *src = a.W + (int64_t)row * a.ldw + a.col0 + grp * 16;
        const half8_t w0 = reinterpret_cast<const half8_t *>(src)[0], w1 = reinterpret_cast<const half8_t *>(src)[1];
        uint64_t out = 0;
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            const float vx = (float)(m < 4 ? w0[2 * m] : w1[2 * m - 8]);
            const float vy = (float)(m < 4 ? w0[2 * m + 1] : w1[2 * m - 7]);
            int best = 0;
            float bd = 3.0e38f;
            for (int c = 0; c < (1 << CB); ++c) {
                const float dx = vx - lx[c], dy = vy - ly[c];
                const float d = dx * dx + dy * dy;
                if (d < bd) { bd = d; best = c; }
            }
            out |= (uint64_t)best << (CB * m);
        }
        uint8_t *dst = a.codes + (int64_t)row * a.row_stride + a.code_off + (int64_t)grp * CB;
#pragma unroll
        for (int b = 0; b < CB; ++b) dst[b] = (uint8_t)(out >> (8 * b));
    }
}

// ------------------------------------------------------------------ trellis
// One workgroup of 1024 threads per tile; thread t keeps the path costs of states
// 64 t .. 64 t + 63 in registers.  A step i: the predecessors of a state st are the F = 2^s
// states (g << s) | f with g = st mod 2^(16-s), consecutive and all owned by one thread, so
// every thread reduces its 64 costs to 64 / F group minima (decision f kept, one byte per
// group and step, in the workspace), the minima travel through LDS (stored transposed, so that
// a thread's 64 reads and its neighbours' fall into different banks), and every thread adds
// the distance of its own 64 states to step i's targets.  Constant terms |v|^2 are left out
// of the costs and added at the end.
// With more than 6 bits per step a group's 2^s predecessors span 2^(s-6) neighbouring threads
// (all 64 states of a thread then belong to one group): the group minimum is finished with
// wavefront shuffles and the decision needs more than a byte from s = 9 on.
template <int SB> struct QpDecision { typedef uint8_t type; };
template <> struct QpDecision<9> { typedef uint16_t type; };
template <> struct QpDecision<10> { typedef uint16_t type; };

template <int V, int SB, int TB>
__global__ __launch_bounds__(1024) void k_encode_trellis(QpEnc a, int tiles_per_row, int64_t ntiles) {
    typedef typename QpDecision<SB>::type dec_t;
    constexpr int n = 256 / V;          // steps per tile
    constexpr int F = 1 << SB;          // values of the s fresh bits
    constexpr int G = 65536 >> SB;      // groups = values of the 16 - s shared bits
    constexpr int GPT = (F <= 64) ? 64 / F : 1;   // groups per thread (F <= 64)
    constexpr int NL = (F <= 64) ? 1 : F / 64;    // threads per group (F > 64)
    constexpr int TP = G / 64;          // group g = 64 t' + k lives at [k][t'], t' < TP
    constexpr int TPP = TP + 1;
    constexpr uint32_t LOW = G - 1;
    constexpr int HALF = n / 2;
    constexpr int NW = (n * SB + 31) / 32;   // dwords of a tile's stream
    __shared__ float gm[2][64 * TPP];
    constexpr int TLN = 2 << TB;        // hybrid code book with the sign folded in
    __shared__ uint32_t tl[V == 2 ? TLN : 1];
    __shared__ __attribute__((aligned(16))) half_t vt[256];
    __shared__ uint16_t states[n];
    __shared__ float redv[16];
    __shared__ uint32_t redi[16];
    __shared__ uint32_t sh_overlap;
    __shared__ float sh_best;
    __shared__ uint32_t outw[NW];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int tq = t & (TP - 1);
    const uint32_t st0 = 64u * t;
    dec_t *back = reinterpret_cast<dec_t *>(a.back) + (size_t)blockIdx.x * n * G;

    // the values of this thread's 64 states
    uint32_t lv1[V == 1 ? 32 : 1];   // two fp16 values per register
    if constexpr (V == 1) {
        const u32x4_t *src = reinterpret_cast<const u32x4_t *>(a.lut + st0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const u32x4_t h = src[c];
#pragma unroll
            for (int e = 0; e < 4; ++e) lv1[4 * c + e] = h[e];
        }
    } else {
        // hybrid code book (App. C.3.1): 2^(TB+1) entries, the upper half with component 0 negated
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a.lut);
        for (int e = t; e < TLN; e += 1024) tl[e] = src[e & ((1 << TB) - 1)] ^ ((uint32_t)(e >> TB) << 15);
    }
    __syncthreads();

    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int row = (int)(tile / tiles_per_row), c = (int)(tile - (int64_t)row * tiles_per_row);
        if (t < 32)
            reinterpret_cast<half8_t *>(vt)[t] =
                reinterpret_cast<const half8_t *>(a.W + (int64_t)row * a.ldw + a.col0 + c * 256)[t];
        __syncthreads();

        float cost[64];
        for (int pass = 0; pass < 2; ++pass) {
            const int shift = (pass == 0) ? HALF : 0;   // pass 0 runs over the tile rotated by half its steps
            const uint32_t overlap = sh_overlap;        // meaningful in pass 1 only
            int buf = 0;
            for (int i = 0; i < n; ++i) {
                int iv = i + shift;
                if (iv >= n) iv -= n;
                if (i > 0) {
                    // group minima of the previous step's costs and the decisions
                    if constexpr (F <= 64) {
                        uint8_t dec[GPT];
#pragma unroll
                        for (int j = 0; j < GPT; ++j) {
                            float bc = cost[j * F];
                            uint32_t bf = 0;
#pragma unroll
                            for (int f = 1; f < F; ++f) {
                                const float cc = cost[j * F + f];
                                if (cc < bc) { bc = cc; bf = f; }
                            }
                            const int g = t * GPT + j;
                            gm[buf][(g & 63) * TPP + (g >> 6)] = bc;
                            dec[j] = (uint8_t)bf;
                        }
                        uint8_t *brow = reinterpret_cast<uint8_t *>(back) + (size_t)i * G + (size_t)t * GPT;
                        if constexpr (GPT >= 4) {
#pragma unroll
                            for (int j4 = 0; j4 < GPT / 4; ++j4)
                                reinterpret_cast<uint32_t *>(brow)[j4] =
                                    (uint32_t)dec[4 * j4] | ((uint32_t)dec[4 * j4 + 1] << 8) |
                                    ((uint32_t)dec[4 * j4 + 2] << 16) | ((uint32_t)dec[4 * j4 + 3] << 24);
                        } else {
#pragma unroll
                            for (int j = 0; j < GPT; ++j) brow[j] = dec[j];
                        }
                    } else {
                        float bc = cost[0];
                        uint32_t bf = 0;
#pragma unroll
                        for (int k = 1; k < 64; ++k)
                            if (cost[k] < bc) { bc = cost[k]; bf = k; }
                        bf += (uint32_t)(t & (NL - 1)) * 64u;
#pragma unroll
                        for (int m = 1; m < NL; m <<= 1) {
                            const float ov = __shfl_xor(bc, m, 64);
                            const uint32_t oi = __shfl_xor(bf, m, 64);
                            if (ov < bc || (ov == bc && oi < bf)) { bc = ov; bf = oi; }
                        }
                        if ((t & (NL - 1)) == 0) {
                            const int g = t / NL;
                            gm[buf][(g & 63) * TPP + (g >> 6)] = bc;
                            back[(size_t)i * G + g] = (dec_t)bf;
                        }
                    }
                    __syncthreads();
                }
                // distances of this thread's states to step i's targets
                float m2v = 0.f;
                half2v m2v2 = half2v{0, 0};
                if constexpr (V == 1) m2v = -2.0f * (float)vt[iv];
                else m2v2 = half2v{(half_t)(-2.0f * (float)vt[2 * iv]), (half_t)(-2.0f * (float)vt[2 * iv + 1])};
                // In chunks of eight states, fenced for the instruction scheduler (left alone it
                // starts all 64 LDS reads first), and with the per-state constants hidden from
                // the optimiser behind empty asm statements: hoisted out of the step loop, the
                // 64 converted table values (or hashed table addresses) would not fit the
                // registers next to the 64 costs.
                uint32_t st0i = st0;
                asm volatile("" : "+v"(st0i));
#pragma unroll
                for (int k0 = 0; k0 < 64; k0 += 8) {
#pragma unroll
                    for (int k = k0; k < k0 + 8; ++k) {
                        float base = 0.f;
                        if (i > 0) base = gm[buf][k * TPP + tq];
                        else if (pass == 1 && ((st0 + k) & LOW) != overlap) base = INFINITY;
                        if constexpr (V == 1) {
                            uint32_t pk = lv1[k >> 1];
                            asm volatile("" : "+v"(pk));
                            const float lf = qp_half_bits_to_float((uint16_t)(pk >> (16 * (k & 1))));
                            cost[k] = __builtin_fmaf(lf, lf + m2v, base);
                        } else {
                            const uint32_t st = st0i + k;
                            const uint32_t h = st * (st + 1u);
                            const half2v l2 = __builtin_bit_cast(half2v, tl[(h >> (15 - TB)) & (uint32_t)(TLN - 1)]);
                            cost[k] = __builtin_amdgcn_fdot2(l2, l2, __builtin_amdgcn_fdot2(l2, m2v2, base, false), false);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (i > 0) buf ^= 1;
            }
            // best admissible end state (pass 1: it must wrap onto the fixed bits)
            float bv = INFINITY;
            uint32_t bi = 0;
#pragma unroll
            for (int k = 0; k < 64; ++k) {
                const bool ok = (pass == 0) || (((st0 + k) >> SB) == overlap);
                if (ok && cost[k] < bv) { bv = cost[k]; bi = st0 + k; }
            }
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) {
                const float ov = __shfl_xor(bv, m, 64);
                const uint32_t oi = __shfl_xor(bi, m, 64);
                if (ov < bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (lane == 0) { redv[wave] = bv; redi[wave] = bi; }
            __syncthreads();   // also: every decision byte of this pass is written
            if (t == 0) {
                float b = redv[0];
                uint32_t st = redi[0];
                for (int w = 1; w < 16; ++w)
                    if (redv[w] < b || (redv[w] == b && redi[w] < st)) { b = redv[w]; st = redi[w]; }
                sh_best = b;
                // walk back through the decisions
                const int stop = (pass == 0) ? (n - HALF) : 0;
                for (int i = n - 1; i >= stop; --i) {
                    states[i] = (uint16_t)st;
                    if (i > 0) {
                        const uint32_t g = st & LOW;
                        st = (g << SB) | back[(size_t)i * G + g];
                    }
                }
                // rotated step n - HALF is step 0 of the tile: its low 16 - s bits are the shared bits
                if (pass == 0) sh_overlap = states[n - HALF] & LOW;
            }
            if (pass == 1 && t < NW) outw[t] = 0;
            __syncthreads();
        }
        // lay the states' fresh bits down: step j contributes its low s bits at stream bit j s
        if (t < n) {
            const uint32_t val = states[t] & (F - 1);
            const int bit = t * SB, w = bit >> 5, r = bit & 31;
            atomicOr(&outw[w], val << r);
            if (r + SB > 32) atomicOr(&outw[w + 1], val >> (32 - r));
        }
        __syncthreads();
        uint8_t *dst = a.codes + (int64_t)row * a.row_stride + a.code_off + (int64_t)c * (NW * 4);
        if (t < NW) reinterpret_cast<uint32_t *>(dst)[t] = outw[t];
        if (t == 0 && a.tile_err) {
            float v2 = 0.f;
            for (int e = 0; e < 256; ++e) v2 += (float)vt[e] * (float)vt[e];
            a.tile_err[(int64_t)row * a.tiles_row_total + a.col0 / 256 + c] = sh_best + v2;
        }
        __syncthreads();
    }
}

static size_t trellis_back_bytes(int V, int sb) {
    return (size_t)(256 / V) * (size_t)(65536 >> sb) * (sb > 8 ? 2 : 1);
}

// Workgroups that the trellis encoder runs: one per CU, fewer when the workspace is smaller.
static int trellis_grid(int V, int sb, int64_t ntiles, size_t workspace_bytes) {
    int64_t g = (int64_t)(workspace_bytes / trellis_back_bytes(V, sb));
    if (g > 256) g = 256;
    if (g > ntiles) g = ntiles;
    return (int)g;
}

size_t qp_encode_min_workspace(int scheme, int cb) {
    if (scheme == QP_TCQ) return trellis_back_bytes(1, cb);
    if (scheme == QP_TCQH) return trellis_back_bytes(2, cb);
    if (scheme == QP_TCQHH) return trellis_back_bytes(2, cb);   // the larger of its two halves
    return 0;
}

static qp_status launch_trellis(int V, int sb, int tb, QpEnc a, size_t workspace_bytes, hipStream_t st) {
    const int tiles_per_row = a.ncols / 256;
    const int64_t ntiles = (int64_t)a.M * tiles_per_row;
    const int grid = trellis_grid(V, sb, ntiles, workspace_bytes);
    if (grid < 1) return QP_ERR_WORKSPACE;
#define ENC(VV, SS, TT) \
    hipLaunchKernelGGL((k_encode_trellis<VV, SS, TT>), dim3(grid), dim3(1024), 0, st, a, tiles_per_row, ntiles)
    if (V == 1 && sb == 2) ENC(1, 2, 9);
    else if (V == 1 && sb == 3) ENC(1, 3, 9);
    else if (V == 1 && sb == 4) ENC(1, 4, 9);
    else if (V == 2 && sb == 3 && tb == 9) ENC(2, 3, 9);
    else if (V == 2 && sb == 4 && tb == 9) ENC(2, 4, 9);
    else if (V == 2 && sb == 5 && tb == 9) ENC(2, 5, 9);
    else if (V == 2 && sb == 6 && tb == 9) ENC(2, 6, 9);
    else if (V == 2 && sb == 7 && tb == 9) ENC(2, 7, 9);
    else if (V == 2 && sb == 8 && tb == 9) ENC(2, 8, 9);
    else if (V == 2 && sb == 8 && tb == 10) ENC(2, 8, 10);
    else if (V == 2 && sb == 9 && tb == 10) ENC(2, 9, 10);
    else if (V == 2 && sb == 9 && tb == 11) ENC(2, 9, 11);
    else if (V == 2 && sb == 10 && tb == 11) ENC(2, 10, 11);
    else return QP_ERR_UNSUPPORTED;
#undef ENC
    return qp_check_launch();
}

qp_status qp_launch_encode(int scheme, int cb, int tlut_bits, int M, int N, const uint16_t *lut, const void *W, int64_t ldw,
                           void *codes, int64_t row_stride, void *workspace, size_t workspace_bytes, float *tile_err,
                           hipStream_t st) {
    QpEnc a;
    a.W = static_cast<const half_t *>(W);
    a.ldw = ldw;
    a.M = M;
    a.col0 = 0;
    a.ncols = N;
    a.lut = lut;
    a.codes = static_cast<uint8_t *>(codes);
    a.row_stride = row_stride;
    a.code_off = 0;
    a.back = static_cast<uint8_t *>(workspace);
    a.tile_err = tile_err;
    a.tiles_row_total = N / 256;
    if (scheme == QP_SQ) {
        int64_t total = (int64_t)M * (N / 8);
        int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
        hipLaunchKernelGGL(k_encode_sq4, dim3(blocks), dim3(256), 0, st, a);
        return qp_check_launch();
    }
    if (scheme == QP_VQ) {
        int64_t total = (int64_t)M * (N / 16);
        int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
        if (cb == 5) hipLaunchKernelGGL(k_encode_vq<5>, dim3(blocks), dim3(256), 0, st, a);
        else hipLaunchKernelGGL(k_encode_vq<7>, dim3(blocks), dim3(256), 0, st, a);
        return qp_check_launch();
    }
    if (scheme == QP_TCQ) return launch_trellis(1, cb, 9, a, workspace_bytes, st);
    if (scheme == QP_TCQH) return launch_trellis(2, cb, tlut_bits, a, workspace_bytes, st);
    if (scheme == QP_TCQHH) {
        // two launches on the stream, one per half of the input channels (App. C.3.2 "Quantization")
        a.ncols = N / 2;
        qp_status s = launch_trellis(2, cb, tlut_bits, a, workspace_bytes, st);
        if (s != QP_OK) return s;
        a.col0 = N / 2;
        a.code_off = (int64_t)(N / 512) * (16 * cb);
        return launch_trellis(2, cb + 1, tlut_bits, a, workspace_bytes, st);
    }
    return QP_ERR_UNSUPPORTED;
}

// ------------------------------------------------------------------ per-output-channel scale
// s[j] = sqrt(mean_i W[j, i]^2) rounded to fp16, W[j, :] <- W[j, :] / s[j] (Section 3.3: after
// the rotation the weights of an output channel are divided by their scale so that they are
// close to N(0,1), what the code books are fitted to).  One wavefront per row; a row of zeros
// gets scale 1.
__global__ __launch_bounds__(1024) void k_row_normalize(half_t *W, int64_t ldw, int M, int N, uint16_t *scales) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int row = blockIdx.x * 16 + wave; row < M; row += gridDim.x * 16) {
        half_t *w = W + (int64_t)row * ldw;
        float acc = 0.f;
        for (int i = lane * 8; i < N; i += 512) {
            const half8_t h = *reinterpret_cast<const half8_t *>(w + i);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf((float)h[e], (float)h[e], acc);
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
        half_t s16 = (half_t)sqrtf(acc / (float)N);
        if ((float)s16 == 0.f) s16 = (half_t)1.0f;
        if (lane == 0) scales[row] = __builtin_bit_cast(uint16_t, s16);
        const float inv = 1.0f / (float)s16;
        for (int i = lane * 8; i < N; i += 512) {
            half8_t h = *reinterpret_cast<const half8_t *>(w + i);
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = (half_t)((float)h[e] * inv);
            *reinterpret_cast<half8_t *>(w + i) = h;
        }
    }
}

qp_status qp_launch_row_normalize(void *W, int64_t ldw, int M, int N, void *scales, hipStream_t st) {
    int blocks = (M + 15) / 16;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_row_normalize, dim3(blocks), dim3(1024), 0, st, (half_t *)W, ldw, M, N, (uint16_t *)scales);
    return qp_check_launch();
}
