/*
 * qpo_encode — round-to-nearest encoders of the three quantizer families.
 * TEST INFRASTRUCTURE ONLY (see qpo.c).  The inference path never encodes; these
 * exist so that the decode definitions in qpo.c can be checked as *quantizers*:
 * a decode with a dropped term or a wrong bit order still decodes something, but
 * the distortion an optimal encoder reaches through it no longer meets what the
 * paper and rate-distortion theory fix.
 *
 * Scalar / vector RTN: Appendix C.1 and C.2, "Quantization" (nearest table entry).
 * Trellis RTN: Appendix C.3.1, "Quantization" (the stream whose decode is closest
 * to the target, found with the Viterbi algorithm; tail-biting).
 *
 * All encoders emit the LSB-first packed stream that qpo.c decodes.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

double qpo_half_to_double(uint16_t h);

static void put_bits(uint8_t *stream, int64_t q, int c, uint32_t v)
{
    for (int t = 0; t < c; ++t) {
        int64_t p = q + t;
        if ((v >> t) & 1u) stream[p >> 3] |= (uint8_t)(1u << (p & 7));
        else stream[p >> 3] &= (uint8_t)~(1u << (p & 7));
    }
}

/* Nearest of 2^bits scalar levels; ties go to the lower index. */
void qpo_rtn_sq(const double *v, int64_t n, int bits, const uint16_t *lut, uint8_t *stream)
{
    int K = 1 << bits;
    for (int64_t i = 0; i < n; ++i) {
        int best = 0;
        double bd = DBL_MAX;
        for (int c = 0; c < K; ++c) {
            double d = fabs(v[i] - qpo_half_to_double(lut[c]));
            if (d < bd) { bd = d; best = c; }
        }
        put_bits(stream, i * bits, bits, (uint32_t)best);
    }
}

/* Nearest of 2^cbits V-dimensional points (Euclidean). n counts scalars. */
void qpo_rtn_vq(const double *v, int64_t n, int cbits, int V, const uint16_t *lut, uint8_t *stream)
{
    int K = 1 << cbits;
    for (int64_t m = 0; m < n / V; ++m) {
        int best = 0;
        double bd = DBL_MAX;
        for (int c = 0; c < K; ++c) {
            double d = 0.0;
            for (int u = 0; u < V; ++u) {
                double e = v[m * V + u] - qpo_half_to_double(lut[(int64_t)c * V + u]);
                d += e * e;
            }
            if (d < bd) { bd = d; best = c; }
        }
        put_bits(stream, m * cbits, cbits, (uint32_t)best);
    }
}

/* Squared error between target v[0..T) and the decode of one tile's stream. */
static double tile_error(const double *v, const uint8_t *stream, int s, int L, int T, int V,
                         const double *lut)
{
    int64_t nbits = (int64_t)s * T / V;
    double e = 0.0;
    for (int i = 0; i < T / V; ++i) {
        uint32_t st = 0;
        for (int u = 0; u < L; ++u) {
            int64_t p = ((int64_t)i * s + u) % nbits;
            st |= (uint32_t)((stream[p >> 3] >> (p & 7)) & 1) << u;
        }
        for (int u = 0; u < V; ++u) {
            double d = v[i * V + u] - lut[(int64_t)st * V + u];
            e += d * d;
        }
    }
    return e;
}

/* Exhaustive search over all 2^(sT/V) streams of one tile (tiny tiles only:
 * sT/V <= 24).  Returns the minimum squared error and writes a minimiser. */
double qpo_tcq_encode_brute(const double *v, int s, int L, int T, int V, const uint16_t *lut16,
                            uint8_t *stream)
{
    int nbits = s * T / V;
    int nbytes = (nbits + 7) / 8;
    int64_t nlut = ((int64_t)1 << L) * V;
    double *lut = (double *)malloc(sizeof(double) * (size_t)nlut);
    for (int64_t i = 0; i < nlut; ++i) lut[i] = qpo_half_to_double(lut16[i]);
    uint8_t cand[4] = {0, 0, 0, 0};
    double best = DBL_MAX;
    for (uint32_t w = 0; w < (1u << nbits); ++w) {
        for (int b = 0; b < nbytes; ++b) cand[b] = (uint8_t)(w >> (8 * b));
        double e = tile_error(v, cand, s, L, T, V, lut);
        if (e < best) { best = e; memcpy(stream, cand, (size_t)nbytes); }
    }
    free(lut);
    return best;
}

/*
 * Viterbi over the bitshift trellis.  Step i (0 <= i < n = T/V) is in state
 * state_i = r[i s : i s + L]; the only allowed successors of a state are
 * (state >> s) | (fresh << (L - s)) for the 2^s values of the s fresh bits.
 *
 *   overlap < 0 : open trellis (no tail-biting constraint); the stream written
 *                 is the first n*s bits of the best open path.
 *   overlap >= 0: the L-s bits r[0 : L-s] are fixed to `overlap`, and the last
 *                 state must wrap onto them (state_{n-1} >> s == overlap), which
 *                 is exactly the closed (tail-biting) trellis restricted to one
 *                 value of the bits shared by its two ends.
 * Returns the path's squared error.
 */
static double viterbi_pass(const double *v, int s, int L, int n, int V, const double *lut,
                           int64_t overlap, uint8_t *stream, uint16_t *back /* n * 2^L decisions, up to s = 16 bits each */,
                           double *cost /* 2 * 2^L */)
{
    int64_t S = (int64_t)1 << L;
    int F = 1 << s;
    uint32_t lowmask = (uint32_t)((1u << (L - s)) - 1u);
    double *cur = cost, *nxt = cost + S;
    for (int64_t st = 0; st < S; ++st) {
        double e = 0.0;
        for (int u = 0; u < V; ++u) {
            double d = v[u] - lut[st * V + u];
            e += d * d;
        }
        cur[st] = (overlap >= 0 && ((uint32_t)st & lowmask) != (uint32_t)overlap) ? DBL_MAX : e;
    }
    for (int i = 1; i < n; ++i) {
        for (int64_t st = 0; st < S; ++st) {
            /* predecessors p satisfy p >> s == st & lowmask; their low s bits are free */
            uint32_t base = ((uint32_t)st & lowmask) << s;
            double bc = DBL_MAX;
            int bf = 0;
            for (int f = 0; f < F; ++f) {
                double c = cur[base | (uint32_t)f];
                if (c < bc) { bc = c; bf = f; }
            }
            double e = 0.0;
            for (int u = 0; u < V; ++u) {
                double d = v[i * V + u] - lut[st * V + u];
                e += d * d;
            }
            nxt[st] = (bc == DBL_MAX) ? DBL_MAX : bc + e;
            back[(int64_t)i * S + st] = (uint16_t)bf;
        }
        double *t = cur; cur = nxt; nxt = t;
    }
    /* best admissible end state */
    int64_t end = -1;
    double best = DBL_MAX;
    for (int64_t st = 0; st < S; ++st) {
        if (overlap >= 0 && ((uint32_t)st >> s) != (uint32_t)overlap) continue;
        if (cur[st] < best) { best = cur[st]; end = st; }
    }
    if (end < 0) return DBL_MAX;
    /* walk back: collect the states, then lay their bits down */
    uint32_t *states = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
    uint32_t st = (uint32_t)end;
    for (int i = n - 1; i >= 0; --i) {
        states[i] = st;
        if (i > 0) st = ((st & lowmask) << s) | back[(int64_t)i * S + st];
    }
    /* state_i's low s bits are stream bits [i s, i s + s) */
    for (int i = 0; i < n; ++i) put_bits(stream, (int64_t)i * s, s, states[i] & (uint32_t)(F - 1));
    free(states);
    return best;
}

/* Exact tail-biting encode: one constrained pass per value of the shared bits
 * (2^(L-s) passes) — affordable for small L only. */
double qpo_tcq_encode_viterbi_exact(const double *v, int s, int L, int T, int V,
                                    const uint16_t *lut16, uint8_t *stream)
{
    int n = T / V;
    int64_t S = (int64_t)1 << L;
    int nbytes = (s * n + 7) / 8;
    double *lut = (double *)malloc(sizeof(double) * (size_t)(S * V));
    for (int64_t i = 0; i < S * V; ++i) lut[i] = qpo_half_to_double(lut16[i]);
    uint16_t *back = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n * (size_t)S);
    double *cost = (double *)malloc(sizeof(double) * 2 * (size_t)S);
    uint8_t *cand = (uint8_t *)calloc((size_t)nbytes + 1, 1);
    double best = DBL_MAX;
    for (int64_t o = 0; o < ((int64_t)1 << (L - s)); ++o) {
        memset(cand, 0, (size_t)nbytes);
        double e = viterbi_pass(v, s, L, n, V, lut, o, cand, back, cost);
        if (e < best) { best = e; memcpy(stream, cand, (size_t)nbytes); }
    }
    free(cand); free(cost); free(back); free(lut);
    return best;
}

/* Two-pass tail-biting encode for L = 16: an open pass over the target rotated
 * by half a tile picks the bits that the two ends share, then one constrained
 * pass closes the trellis on them.  Not guaranteed optimal; always returns a
 * valid tail-biting stream.  Returns the squared error *recomputed through the
 * decode definition* (tile_error), not the trellis path metric. */
double qpo_tcq_encode_viterbi(const double *v, int s, int L, int T, int V, const uint16_t *lut16,
                              uint8_t *stream)
{
    int n = T / V;
    int64_t S = (int64_t)1 << L;
    int nbits = s * n;
    int nbytes = (nbits + 7) / 8;
    double *lut = (double *)malloc(sizeof(double) * (size_t)(S * V));
    for (int64_t i = 0; i < S * V; ++i) lut[i] = qpo_half_to_double(lut16[i]);
    uint16_t *back = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n * (size_t)S);
    double *cost = (double *)malloc(sizeof(double) * 2 * (size_t)S);
    double *rot = (double *)malloc(sizeof(double) * (size_t)T);
    uint8_t *tmp = (uint8_t *)calloc((size_t)nbytes + 1, 1);
    int half = n / 2;
    for (int i = 0; i < n; ++i)
        for (int u = 0; u < V; ++u) rot[i * V + u] = v[((i + half) % n) * V + u];
    viterbi_pass(rot, s, L, n, V, lut, -1, tmp, back, cost);
    /* original step 0 is rotated step n - half; its first L-s bits: */
    uint32_t overlap = 0;
    for (int u = 0; u < L - s; ++u) {
        int64_t p = ((int64_t)(n - half) * s + u) % nbits;
        overlap |= (uint32_t)((tmp[p >> 3] >> (p & 7)) & 1) << u;
    }
    memset(stream, 0, (size_t)nbytes);
    viterbi_pass(v, s, L, n, V, lut, (int64_t)overlap, stream, back, cost);
    double e = tile_error(v, stream, s, L, T, V, lut);
    free(tmp); free(rot); free(cost); free(back); free(lut);
    return e;
}

/* Best tail-biting stream among those whose first L - s bits equal `overlap` (one
 * constrained Viterbi pass, exact for that value of the shared bits).  Returns its squared
 * error; DBL_MAX if overlap is out of range.  Used to check an encoder that picked its own
 * value of the shared bits: its result can be no better than this, and should be no worse. */
double qpo_tcq_encode_constrained(const double *v, int s, int L, int T, int V, const uint16_t *lut16,
                                  uint32_t overlap, uint8_t *stream)
{
    int n = T / V;
    int64_t S = (int64_t)1 << L;
    int nbytes = (s * n + 7) / 8;
    if (overlap >> (L - s)) return DBL_MAX;
    double *lut = (double *)malloc(sizeof(double) * (size_t)(S * V));
    for (int64_t i = 0; i < S * V; ++i) lut[i] = qpo_half_to_double(lut16[i]);
    uint16_t *back = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n * (size_t)S);
    double *cost = (double *)malloc(sizeof(double) * 2 * (size_t)S);
    memset(stream, 0, (size_t)nbytes);
    viterbi_pass(v, s, L, n, V, lut, (int64_t)overlap, stream, back, cost);
    double e = tile_error(v, stream, s, L, T, V, lut);
    free(cost); free(back); free(lut);
    return e;
}

/* Squared error of the decode of an arbitrary tile stream against the target. */
double qpo_tcq_tile_error(const double *v, const uint8_t *stream, int s, int L, int T, int V,
                          const uint16_t *lut16)
{
    int64_t S = (int64_t)1 << L;
    double *lut = (double *)malloc(sizeof(double) * (size_t)(S * V));
    for (int64_t i = 0; i < S * V; ++i) lut[i] = qpo_half_to_double(lut16[i]);
    double e = tile_error(v, stream, s, L, T, V, lut);
    free(lut);
    return e;
}

/* Many tiles at once (threads over tiles when built with OpenMP). */
void qpo_tcq_encode_tiles(const double *v, int64_t ntiles, int s, int L, int T, int V,
                          const uint16_t *lut16, uint8_t *streams, double *errs)
{
    int64_t tile_bytes = (int64_t)s * T / V / 8;
#if defined(_OPENMP)
#pragma omp parallel for schedule(dynamic)
#endif
    for (int64_t t = 0; t < ntiles; ++t)
        errs[t] = qpo_tcq_encode_viterbi(v + t * T, s, L, T, V, lut16, streams + t * tile_bytes);
}
