/*
 * qpo — plain CPU oracle for the quantized-linear hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct statement of what the path computes,
 * written from the paper's definitions.  It shares no code, header, table or
 * helper with the GPU library and must never be linked into, imported by or
 * called from the product path: only the tests, the smoke check and the
 * benchmark's "cpu_baseline" leg may use it.
 *
 * Everything floating point is IEEE binary64.  fp16 inputs are converted
 * exactly (every binary16 value is representable in binary64).  There is no
 * blocking, fusion or reordering: loops run in index order.
 *
 * Conventions fixed here because the paper leaves them open (they are the
 * definition both sides of a parity test implement):
 *   - a bitstream is a byte array; stream bit p is bit (p mod 8) of byte
 *     floor(p/8)  (LSB first);
 *   - a c-bit code that starts at stream bit q has value sum_t bit(q+t) 2^t;
 *   - weights are stored row by row: row j of W^ (output channel j) is one
 *     stream of N weights along the input dimension;
 *   - a trellis tile is T consecutive input channels of one output row, the
 *     tiles of a row follow each other, and the sliding window wraps inside
 *     its own tile (tail-biting).
 *
 * Parity pins (tests/test_oracle_*.py): exhaustive fp16 conversion against
 * numpy; decode against numpy.take on independently unpacked indices and
 * against single-bit / all-zero / all-one streams; trellis decode against the
 * L = k special case (which is scalar decode) and against the shift-register
 * recurrence; Hadamard against H H^T = n I, Parseval, involution and the
 * fast transform below; matmul against numpy float64; the encoders against
 * exhaustive search on tiny trellises and the Gaussian distortion-rate bound
 * and the paper's printed NUQ-2 distortion (Appendix A, distortion table).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#if defined(_OPENMP)
#include <omp.h>
#endif

/* ------------------------------------------------------------------ fp16 */

/* Exact value of an IEEE binary16 bit pattern. */
double qpo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);                 /* zero and subnormals */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp((double)(frac | 0x400), expo - 25); /* 1.f * 2^(e-15) */
    return sign ? -v : v;
}

void qpo_half_to_double_array(const uint16_t *h, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = qpo_half_to_double(h[i]);
}

/* ------------------------------------------------------------ bit access */

int qpo_bit(const uint8_t *stream, int64_t p)
{
    return (stream[p >> 3] >> (p & 7)) & 1;
}

/* c-bit code starting at stream bit q (no wrap). */
uint32_t qpo_code(const uint8_t *stream, int64_t q, int c)
{
    uint32_t v = 0;
    for (int t = 0; t < c; ++t) v |= (uint32_t)qpo_bit(stream, q + t) << t;
    return v;
}

/* L-bit window starting at bit q of a circular stream of nbits bits. */
uint32_t qpo_window(const uint8_t *stream, int64_t q, int L, int64_t nbits)
{
    uint32_t v = 0;
    for (int u = 0; u < L; ++u) v |= (uint32_t)qpo_bit(stream, (q + u) % nbits) << u;
    return v;
}

/* ------------------------------------------------- decode: one row each */

/* Scalar quantizer (Appendix C.1, "Dequantization"): W^[i] = LUT[int(r_i)],
 * r_i the i-th b-bit code of the row. */
void qpo_decode_row_sq(const uint8_t *row, int N, int bits, const uint16_t *lut, uint16_t *out)
{
    for (int i = 0; i < N; ++i) out[i] = lut[qpo_code(row, (int64_t)i * bits, bits)];
}

/* 2-D vector quantizer (Appendix C.2, "Dequantization"): the m-th c-bit code
 * of the row selects LUT[idx] in R^2, whose components are columns 2m, 2m+1.
 * Written for general V. */
void qpo_decode_row_vq(const uint8_t *row, int N, int cbits, int V, const uint16_t *lut, uint16_t *out)
{
    for (int m = 0; m < N / V; ++m) {
        uint32_t idx = qpo_code(row, (int64_t)m * cbits, cbits);
        for (int v = 0; v < V; ++v) out[m * V + v] = lut[(int64_t)idx * V + v];
    }
}

/* Bitshift trellis with tail-biting (Section 3.2 "Trellis-coded quantization";
 * Appendix C.3.1 "Dequantization"): inside one tile with bit array r of length
 * s*T/V, the i-th V-subvector is LUT[ r[i*s : i*s+L] ], indices taken modulo
 * the tile's length. */
void qpo_decode_row_tcq(const uint8_t *row, int N, int s, int L, int T, int V,
                        const uint16_t *lut, uint16_t *out)
{
    int64_t tile_bits = (int64_t)s * T / V;
    int64_t tile_bytes = tile_bits / 8;
    for (int t = 0; t < N / T; ++t) {
        const uint8_t *r = row + t * tile_bytes;
        for (int i = 0; i < T / V; ++i) {
            uint32_t state = qpo_window(r, (int64_t)i * s, L, tile_bits);
            for (int v = 0; v < V; ++v)
                out[(int64_t)t * T + i * V + v] = lut[(int64_t)state * V + v];
        }
    }
}

/* The same trellis decode written as a shift register: the state is read in
 * full once, then every step drops its s oldest bits and takes s new ones at
 * the top.  A second implementation used only to cross-check the one above. */
void qpo_decode_row_tcq_recurrence(const uint8_t *row, int N, int s, int L, int T, int V,
                                   const uint16_t *lut, uint16_t *out)
{
    int64_t tile_bits = (int64_t)s * T / V;
    int64_t tile_bytes = tile_bits / 8;
    uint32_t mask = (L == 32) ? 0xffffffffu : ((1u << L) - 1u);
    for (int t = 0; t < N / T; ++t) {
        const uint8_t *r = row + t * tile_bytes;
        uint32_t state = qpo_window(r, 0, L, tile_bits);
        for (int i = 0; i < T / V; ++i) {
            for (int v = 0; v < V; ++v)
                out[(int64_t)t * T + i * V + v] = lut[(int64_t)state * V + v];
            uint32_t fresh = qpo_window(r, (int64_t)i * s + L, s, tile_bits);
            state = ((state >> s) | (fresh << (L - s))) & mask;
        }
    }
}

/* Hybrid computed code book of the trellis quantizer (Appendix C.3.1, "Codebook
 * construction"): the 2^16 x 2 table is not stored but derived from a small table
 * tlut[2^tb][2].  For a 16-bit state x, with h = x (x + 1) (no overflow: h < 2^32),
 *   - the tb bits of h just below bit 15 select the entry,  idx = (h >> (15 - tb)) mod 2^tb,
 *   - bit 15 of h negates component 0 of that entry.
 * lut receives the expanded table, fp16 patterns [65536][2]. */
void qpo_hybrid_lut(const uint16_t *tlut, int tb, uint16_t *lut)
{
    for (uint32_t x = 0; x < 65536u; ++x) {
        uint64_t h = (uint64_t)x * ((uint64_t)x + 1u);
        uint32_t idx = (uint32_t)((h >> (15 - tb)) & ((1u << tb) - 1u));
        int negate = (int)((h >> 15) & 1u);
        uint16_t c0 = tlut[2 * idx], c1 = tlut[2 * idx + 1];
        lut[2 * x] = negate ? (uint16_t)(c0 ^ 0x8000u) : c0;   /* fp16 negation = sign bit */
        lut[2 * x + 1] = c1;
    }
}

/* Half-TCQ (Section 3.2; Appendix C.3.2 "Dequantization"): the input channels are cut in
 * two halves; the first N/2 weights of a row are a trellis stream with s bits per step,
 * the second N/2 a trellis stream with s + 1 bits per step (bitwidths b and b + 1/2 at
 * V = 2), both decoded with the same table, and the two decoded halves are concatenated.
 * The second stream starts at the byte after the first one's last tile. */
void qpo_decode_row_half_tcq(const uint8_t *row, int N, int s, int L, int T, int V,
                             const uint16_t *lut, uint16_t *out)
{
    int half = N / 2;
    int64_t first_bytes = (int64_t)(half / T) * ((int64_t)s * T / V / 8);
    qpo_decode_row_tcq(row, half, s, L, T, V, lut, out);
    qpo_decode_row_tcq(row + first_bytes, half, s + 1, L, T, V, lut, out + half);
}

enum { QPO_SQ = 0, QPO_VQ = 1, QPO_TCQ = 2, QPO_HALF_TCQ = 3 };

static void decode_row(int scheme, const uint8_t *row, int N, int code_bits, int V, int L, int T,
                       const uint16_t *lut, uint16_t *out)
{
    if (scheme == QPO_SQ) qpo_decode_row_sq(row, N, code_bits, lut, out);
    else if (scheme == QPO_VQ) qpo_decode_row_vq(row, N, code_bits, V, lut, out);
    else if (scheme == QPO_HALF_TCQ) qpo_decode_row_half_tcq(row, N, code_bits, L, T, V, lut, out);
    else qpo_decode_row_tcq(row, N, code_bits, L, T, V, lut, out);
}

/* Whole matrix: out is uint16 [M, N] row-major, the unscaled fp16 patterns. */
int qpo_decode(int scheme, const uint8_t *codes, int64_t row_stride, int M, int N,
               int code_bits, int V, int L, int T, const uint16_t *lut, uint16_t *out)
{
    if (scheme < 0 || scheme > 3) return 1;
    for (int j = 0; j < M; ++j)
        decode_row(scheme, codes + (int64_t)j * row_stride, N, code_bits, V, L, T, lut,
                   out + (int64_t)j * N);
    return 0;
}

/* ----------------------------------------------------------- Hadamard */

/* Sylvester matrix entry: H_1 = [1], H_2m = [[H,H],[H,-H]]  =>
 * H[a][b] = (-1)^popcount(a & b). */
int qpo_hadamard_entry(uint32_t a, uint32_t b)
{
    uint32_t x = a & b;
    int p = 0;
    while (x) { p ^= (int)(x & 1u); x >>= 1; }
    return p ? -1 : 1;
}

/* Randomized block Hadamard rotation of each row of x (Section 3.3, online
 * rotation X -> X R): for every contiguous block of `block` entries,
 *     out_block = H_block (sigma .* x)_block / sqrt(block),
 * evaluated as the dense matrix-vector product.  x is fp16 [B, ldx]; out is
 * double [B, n]. */
void qpo_hadamard_dense(const uint16_t *x, const int8_t *signs, int B, int n, int block,
                        int64_t ldx, double *out)
{
    double norm = 1.0 / sqrt((double)block);
    for (int b = 0; b < B; ++b)
        for (int q = 0; q < n / block; ++q)
            for (int a = 0; a < block; ++a) {
                double acc = 0.0;
                for (int c = 0; c < block; ++c) {
                    double v = (double)signs[q * block + c] * qpo_half_to_double(x[b * ldx + q * block + c]);
                    acc += (double)qpo_hadamard_entry((uint32_t)a, (uint32_t)c) * v;
                }
                out[(int64_t)b * n + q * block + a] = acc * norm;
            }
}

/* Second implementation (butterflies), used only to cross-check the dense one
 * and to make the big chained checks affordable. */
void qpo_hadamard_fast(const uint16_t *x, const int8_t *signs, int B, int n, int block,
                       int64_t ldx, double *out)
{
    double norm = 1.0 / sqrt((double)block);
    for (int b = 0; b < B; ++b)
        for (int q = 0; q < n / block; ++q) {
            double *o = out + (int64_t)b * n + q * block;
            for (int c = 0; c < block; ++c)
                o[c] = (double)signs[q * block + c] * qpo_half_to_double(x[b * ldx + q * block + c]);
            for (int h = 1; h < block; h <<= 1)
                for (int i = 0; i < block; i += 2 * h)
                    for (int j = i; j < i + h; ++j) {
                        double u = o[j], v = o[j + h];
                        o[j] = u + v;
                        o[j + h] = u - v;
                    }
            for (int c = 0; c < block; ++c) o[c] *= norm;
        }
}

/* -------------------------------------------------------------- matmul */

/* y[b][j] = s[j] * sum_i x[b][i] W[j][i], all binary64, index order.
 * x double [B, N], W fp16 patterns [M, N], s fp16 [M], y double [B, M]. */
void qpo_matmul_scaled(const double *x, const uint16_t *W, const uint16_t *s, int B, int M, int N,
                       double *y)
{
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < M; ++j) {
            double acc = 0.0;
            for (int i = 0; i < N; ++i)
                acc += x[(int64_t)b * N + i] * qpo_half_to_double(W[(int64_t)j * N + i]);
            y[(int64_t)b * M + j] = qpo_half_to_double(s[j]) * acc;
        }
}

/* The fused layer as the paper states it: decode row j, take its dot product
 * with every activation row, scale by the per-output-channel factor.
 * x is double [B, N] (the rotated activations, exact values of whatever the
 * caller holds); y is double [B, M].  rows [row_begin, row_end) only, so that
 * a sampled subset of a big layer can be checked.  With OpenMP the loop over
 * output rows is shared between threads; each row's arithmetic is unchanged. */
int qpo_linear_rows(int scheme, const uint8_t *codes, int64_t row_stride, int M, int N,
                    int code_bits, int V, int L, int T, const uint16_t *lut, const uint16_t *scales,
                    const double *x, int B, int row_begin, int row_end, double *y, int use_threads)
{
    if (scheme < 0 || scheme > 3) return 1;
    (void)use_threads;
#if defined(_OPENMP)
#pragma omp parallel if (use_threads)
#endif
    {
        uint16_t *w = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)N);
#if defined(_OPENMP)
#pragma omp for schedule(static)
#endif
        for (int j = row_begin; j < row_end; ++j) {
            decode_row(scheme, codes + (int64_t)j * row_stride, N, code_bits, V, L, T, lut, w);
            double sj = qpo_half_to_double(scales[j]);
            for (int b = 0; b < B; ++b) {
                double acc = 0.0;
                for (int i = 0; i < N; ++i) acc += x[(int64_t)b * N + i] * qpo_half_to_double(w[i]);
                y[(int64_t)b * M + j] = sj * acc;
            }
        }
        free(w);
    }
    return 0;
}

int qpo_num_threads(void)
{
#if defined(_OPENMP)
    return omp_get_max_threads();
#else
    return 1;
#endif
}
