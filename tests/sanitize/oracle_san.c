/* Drives every function of the CPU oracle on small inputs held in exactly-sized heap buffers, so that a
 * build with -fsanitize=address,undefined reports any read or write past an operand, any signed overflow,
 * misaligned access or bad shift.  Values are not checked here (the pins do that); this program only has
 * to run to the end.  Built and run by tests/test_host_sanitizers.py. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double qpo_half_to_double(uint16_t h);
void qpo_half_to_double_array(const uint16_t *h, int64_t n, double *out);
int qpo_bit(const uint8_t *stream, int64_t p);
uint32_t qpo_code(const uint8_t *stream, int64_t q, int c);
uint32_t qpo_window(const uint8_t *stream, int64_t q, int L, int64_t nbits);
void qpo_hybrid_lut(const uint16_t *tlut, int tb, uint16_t *lut);
int qpo_decode(int scheme, const uint8_t *codes, int64_t row_stride, int M, int N, int code_bits, int V, int L, int T,
               const uint16_t *lut, uint16_t *out);
void qpo_decode_row_tcq_recurrence(const uint8_t *row, int N, int s, int L, int T, int V, const uint16_t *lut, uint16_t *out);
int qpo_hadamard_entry(uint32_t a, uint32_t b);
void qpo_hadamard_dense(const uint16_t *x, const int8_t *signs, int B, int n, int block, int64_t ldx, double *out);
void qpo_hadamard_fast(const uint16_t *x, const int8_t *signs, int B, int n, int block, int64_t ldx, double *out);
void qpo_matmul_scaled(const double *x, const uint16_t *W, const uint16_t *s, int B, int M, int N, double *y);
int qpo_linear_rows(int scheme, const uint8_t *codes, int64_t row_stride, int M, int N, int code_bits, int V, int L, int T,
                    const uint16_t *lut, const uint16_t *scales, const double *x, int B, int row_begin, int row_end,
                    double *y, int use_threads);
void qpo_rtn_sq(const double *v, int64_t n, int bits, const uint16_t *lut, uint8_t *stream);
void qpo_rtn_vq(const double *v, int64_t n, int cbits, int V, const uint16_t *lut, uint8_t *stream);
double qpo_tcq_encode_brute(const double *v, int s, int L, int T, int V, const uint16_t *lut16, uint8_t *stream);
double qpo_tcq_encode_viterbi_exact(const double *v, int s, int L, int T, int V, const uint16_t *lut16, uint8_t *stream);
double qpo_tcq_encode_viterbi(const double *v, int s, int L, int T, int V, const uint16_t *lut16, uint8_t *stream);
double qpo_tcq_encode_constrained(const double *v, int s, int L, int T, int V, const uint16_t *lut16, uint32_t overlap,
                                  uint8_t *stream);
double qpo_tcq_tile_error(const double *v, const uint8_t *stream, int s, int L, int T, int V, const uint16_t *lut16);
void qpo_tcq_encode_tiles(const double *v, int64_t ntiles, int s, int L, int T, int V, const uint16_t *lut16,
                          uint8_t *streams, double *errs);
double qpo_kmeans_assign(const double *x, int64_t n, int d, const double *m, int k, int32_t *a);
double qpo_kmeans_update(const double *x, int64_t n, int d, const int32_t *a, const double *m_in, int k, double *m_out,
                         int64_t *count);
int qpo_kmeans(const double *x, int64_t n, int d, double *m, int k, int max_iter, double tol, double *inertia);

static uint32_t rs = 12345u;
static uint32_t rnd(void) { rs = rs * 1664525u + 1013904223u; return rs >> 8; }
static uint16_t rnd_half(void) { return (uint16_t)(0x3000u + (rnd() & 0x0fffu)) | (uint16_t)((rnd() & 1u) << 15); }   /* a finite fp16 */
static void *buf(size_t n) { void *p = malloc(n ? n : 1); if (!p) exit(2); return p; }
static uint8_t *rnd_bytes(size_t n) { uint8_t *p = buf(n); for (size_t i = 0; i < n; ++i) p[i] = (uint8_t)rnd(); return p; }
static uint16_t *rnd_halves(size_t n) { uint16_t *p = buf(2 * n); for (size_t i = 0; i < n; ++i) p[i] = rnd_half(); return p; }
static double *rnd_doubles(size_t n) { double *p = buf(8 * n); for (size_t i = 0; i < n; ++i) p[i] = ((int)(rnd() % 2001) - 1000) / 500.0; return p; }

/* decode + fused layer of one scheme; row_bytes is the exact length of a row */
static void layer(int scheme, int M, int N, int cb, int V, int L, int T, size_t lut_halves, size_t row_bytes)
{
    uint8_t *codes = rnd_bytes((size_t)M * row_bytes);
    uint16_t *lut = rnd_halves(lut_halves), *scales = rnd_halves((size_t)M), *out = buf(2 * (size_t)M * N);
    double *x = rnd_doubles(3 * (size_t)N), *y = buf(8 * 3 * (size_t)M);
    if (qpo_decode(scheme, codes, (int64_t)row_bytes, M, N, cb, V, L, T, lut, out)) exit(3);
    if (qpo_linear_rows(scheme, codes, (int64_t)row_bytes, M, N, cb, V, L, T, lut, scales, x, 3, 0, M, y, 1)) exit(3);
    if (qpo_linear_rows(scheme, codes, (int64_t)row_bytes, M, N, cb, V, L, T, lut, scales, x, 3, 1, M - 1, y, 0)) exit(3);
    qpo_matmul_scaled(x, out, scales, 3, M, N, y);
    if (scheme == 2) qpo_decode_row_tcq_recurrence(codes, N, cb, L, T, V, lut, out);
    free(codes); free(lut); free(scales); free(out); free(x); free(y);
}

int main(void)
{
    /* bit fields at the very end of a stream */
    uint8_t *two = rnd_bytes(2);
    (void)qpo_bit(two, 15); (void)qpo_code(two, 9, 7); (void)qpo_window(two, 13, 16, 16);
    free(two);
    uint16_t *h = rnd_halves(65536); double *hd = buf(8 * 65536);
    for (uint32_t i = 0; i < 65536u; ++i) h[i] = (uint16_t)i;
    qpo_half_to_double_array(h, 65536, hd); (void)qpo_half_to_double(0xfc00);
    free(h); free(hd);
    /* scalar 4 bit; pairs at 5 and 7 bits with rows that end inside a byte (N = 104: 260 bits, N = 120: 420 bits) */
    layer(0, 5, 1024, 4, 1, 0, 0, 16, 512);
    layer(1, 4, 104, 5, 2, 0, 0, 64, 33);
    layer(1, 4, 120, 7, 2, 0, 0, 256, 53);
    layer(1, 3, 1024, 5, 2, 0, 0, 64, 320);
    /* trellis, V = 1 (2^16 entries) and V = 2 (2^16 pairs), the hybrid table expanded first; half-TCQ */
    layer(2, 3, 512, 2, 1, 16, 256, 65536, 128);
    layer(2, 3, 512, 3, 1, 16, 256, 65536, 192);
    for (int tb = 9; tb <= 11; ++tb) {
        uint16_t *tl = rnd_halves((size_t)2 << tb), *big = buf(2 * 2 * 65536);
        qpo_hybrid_lut(tl, tb, big);
        free(tl); free(big);
    }
    layer(2, 3, 512, 5, 2, 16, 256, 2 * 65536, 160);
    layer(2, 2, 256, 10, 2, 16, 256, 2 * 65536, 160);
    layer(3, 3, 2048, 4, 2, 16, 256, 2 * 65536, 1024 / 2 * 4 / 8 + 1024 / 2 * 5 / 8);
    /* rotation: both forms, strided input */
    {
        const int B = 2, n = 3072, ldx = 3080;
        uint16_t *x = rnd_halves((size_t)(B - 1) * ldx + n); int8_t *sg = buf((size_t)n); double *o = buf(8 * (size_t)B * n);
        for (int i = 0; i < n; ++i) sg[i] = (rnd() & 1) ? 1 : -1;
        qpo_hadamard_dense(x, sg, B, n, 1024, ldx, o); qpo_hadamard_fast(x, sg, B, n, 1024, ldx, o);
        qpo_hadamard_fast(x, sg, B, n, 2, ldx, o); (void)qpo_hadamard_entry(0xffffffffu, 0x80000001u);
        free(x); free(sg); free(o);
    }
    /* encoders */
    {
        uint16_t *lut = rnd_halves(16), *lut2 = rnd_halves(64); double *v = rnd_doubles(104);
        uint8_t *s1 = buf(52), *s2 = buf(33);
        qpo_rtn_sq(v, 104, 4, lut, s1); qpo_rtn_vq(v, 104, 5, 2, lut2, s2);
        free(lut); free(lut2); free(v); free(s1); free(s2);
    }
    {
        /* a short trellis that exhaustive search can do (L = 8, T = 8, 2 bits per step), then the real one */
        uint16_t *small = rnd_halves(256); double *v = rnd_doubles(8); uint8_t *st = buf(2);
        (void)qpo_tcq_encode_brute(v, 2, 8, 8, 1, small, st); (void)qpo_tcq_encode_viterbi_exact(v, 2, 8, 8, 1, small, st);
        (void)qpo_tcq_encode_viterbi(v, 2, 8, 8, 1, small, st); (void)qpo_tcq_encode_constrained(v, 2, 8, 8, 1, small, 5u, st);
        (void)qpo_tcq_tile_error(v, st, 2, 8, 8, 1, small);
        free(small); free(v); free(st);
        uint16_t *lut = rnd_halves(65536), *lut2 = rnd_halves(2 * 65536); double *w = rnd_doubles(2 * 256), errs[2];
        uint8_t *t1 = buf(2 * 64), *t2 = buf(2 * 160);
        qpo_tcq_encode_tiles(w, 2, 2, 16, 256, 1, lut, t1, errs);
        qpo_tcq_encode_tiles(w, 2, 10, 16, 256, 2, lut2, t2, errs);
        (void)qpo_tcq_tile_error(w, t2, 10, 16, 256, 2, lut2);
        free(lut); free(lut2); free(w); free(t1); free(t2);
    }
    {
        const int n = 200, d = 2, k = 7;
        double *x = rnd_doubles((size_t)n * d), *m = rnd_doubles((size_t)k * d), *m2 = buf(8 * (size_t)k * d), inertia;
        int32_t *a = buf(4 * (size_t)n); int64_t *cnt = buf(8 * (size_t)k);
        (void)qpo_kmeans_assign(x, n, d, m, k, a); (void)qpo_kmeans_update(x, n, d, a, m, k, m2, cnt);
        (void)qpo_kmeans(x, n, d, m, k, 20, 1e-9, &inertia);
        free(x); free(m); free(m2); free(a); free(cnt);
    }
    puts("oracle: clean");
    return 0;
}
