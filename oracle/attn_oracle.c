/*
 * fp64 CPU oracle for fused multi-head attention forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU kernel is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path.
 *
 * What it computes (the paper only names the operation, in its Introduction
 * and in Table 2, so the definition is the textbook one):
 *
 *   for every batch b, head h and query row i
 *       J      = {0..S-1}            (non-causal)
 *              = {0..i}              (causal, diagonal included)
 *       s_j    = scale * sum_d q[i,d] * k[j,d]
 *       m      = max_{j in J} s_j
 *       l      = sum_{j in J} exp(s_j - m)
 *       lse_i  = m + ln(l)
 *       O[i,:] = (1/l) * sum_{j in J} exp(s_j - m) * v[j,:]
 *
 * q, k, v are [B,H,S,D] contiguous (D fastest) arrays of 16-bit patterns,
 * IEEE binary16 (dtype 0) or bfloat16 (dtype 1); each is widened exactly to
 * double before any arithmetic.  Two passes per row, no tiling, no running
 * rescale, no reordering beyond the loops written here.
 *
 * A second routine, attn_bruteforce, materialises the whole S x S weight
 * matrix in long double WITHOUT subtracting the row maximum (valid only for
 * small logits) so that the two share no numerical trick; it exists to pin
 * the first on tiny shapes.
 *
 * Every function here is pinned by tests/test_oracle_pins.py (closed forms,
 * invariants, brute force, a library softmax); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- exact widening of 16-bit patterns ------------------------------------------------ */

static double widen_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double x;
    if (expo == 0)
        x = ldexp((double)frac, -24);                 /* zero and subnormals: frac * 2^-24 */
    else if (expo == 31)
        x = frac ? NAN : INFINITY;
    else
        x = ldexp((double)(frac | 0x400), expo - 25); /* (1024+frac) * 2^(expo-15-10) */
    return sign ? -x : x;
}

static double widen_bf16(uint16_t h)
{
    /* bfloat16 is the upper half of an IEEE binary32 */
    uint32_t bits = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double widen(uint16_t h, int dtype) { return dtype == 0 ? widen_f16(h) : widen_bf16(h); }

/* exported so the tests can pin the decoders against hand-written bit patterns */
double oracle_widen(unsigned int bits16, int dtype) { return widen((uint16_t)bits16, dtype); }

/* ---- the definition -------------------------------------------------------------------- */

/*
 * Attention for a chosen set of query rows, for every (b,h).
 *   rows[nrows]            query-row indices in [0,S)
 *   o   [B*H, nrows, D]    fp64 out
 *   lse [B*H, nrows]       fp64 out, natural log
 * Returns 0, or -1 on a bad argument or when memory runs out (o and lse are then not to be used).
 */
int attn_oracle_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                     int B, int H, int S, int D, int causal, double scale, int dtype,
                     const int *rows, int nrows, double *o, double *lse)
{
    if (!q || !k || !v || !o || !lse || !rows) return -1;
    if (B <= 0 || H <= 0 || S <= 0 || D <= 0 || nrows < 0) return -1;
    if (dtype != 0 && dtype != 1) return -1;
    for (int r = 0; r < nrows; ++r)
        if (rows[r] < 0 || rows[r] >= S) return -1;

    const long BH = (long)B * H;
    int out_of_memory = 0;   /* set by any thread whose work buffers could not be had */
#pragma omp parallel
    {
        double *kd = malloc(sizeof(double) * (size_t)S * D);   /* one head of K, widened */
        double *vd = malloc(sizeof(double) * (size_t)S * D);
        double *s  = malloc(sizeof(double) * (size_t)S);
        double *qd = malloc(sizeof(double) * (size_t)D);
        const int have = kd && vd && s && qd;
        if (!have) {
#pragma omp atomic write
            out_of_memory = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long bh = 0; bh < BH; ++bh) {
            if (!have) continue;   /* the call fails as a whole, see below */
            const uint16_t *qh = q + (size_t)bh * S * D;
            const uint16_t *kh = k + (size_t)bh * S * D;
            const uint16_t *vh = v + (size_t)bh * S * D;
            for (size_t e = 0; e < (size_t)S * D; ++e) {
                kd[e] = widen(kh[e], dtype);
                vd[e] = widen(vh[e], dtype);
            }
            for (int r = 0; r < nrows; ++r) {
                const int i = rows[r];
                const int nj = causal ? i + 1 : S;          /* keys 0..nj-1 are visible */
                for (int d = 0; d < D; ++d) qd[d] = widen(qh[(size_t)i * D + d], dtype);

                double m = -INFINITY;
                for (int j = 0; j < nj; ++j) {
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d) dot += qd[d] * kd[(size_t)j * D + d];
                    s[j] = scale * dot;
                    if (s[j] > m) m = s[j];
                }
                double l = 0.0;
                for (int j = 0; j < nj; ++j) {
                    s[j] = exp(s[j] - m);
                    l += s[j];
                }
                double *orow = o + ((size_t)bh * nrows + r) * D;
                for (int d = 0; d < D; ++d) orow[d] = 0.0;
                for (int j = 0; j < nj; ++j)
                    for (int d = 0; d < D; ++d) orow[d] += s[j] * vd[(size_t)j * D + d];
                for (int d = 0; d < D; ++d) orow[d] /= l;
                lse[(size_t)bh * nrows + r] = m + log(l);
            }
        }
        free(kd); free(vd); free(s); free(qd);
    }
    return out_of_memory ? -1 : 0;
}

/* All rows: o [B,H,S,D], lse [B,H,S]. */
int attn_oracle(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                int B, int H, int S, int D, int causal, double scale, int dtype,
                double *o, double *lse)
{
    if (S <= 0) return -1;
    int *rows = malloc(sizeof(int) * (size_t)S);
    if (!rows) return -1;
    for (int i = 0; i < S; ++i) rows[i] = i;
    int rc = attn_oracle_rows(q, k, v, B, H, S, D, causal, scale, dtype, rows, S, o, lse);
    free(rows);
    return rc;
}

/*
 * Brute-force twin for tiny shapes: P = exp(scale * Q K^T) with masked entries
 * set to 0, no max subtraction, long double throughout; P is returned too
 * (p [B,H,S,S], fp64) so the tests can look at the weights themselves.
 */
int attn_bruteforce(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                    int B, int H, int S, int D, int causal, double scale, int dtype,
                    double *o, double *lse, double *p)
{
    if (!q || !k || !v || !o || !lse || !p) return -1;
    if (B <= 0 || H <= 0 || S <= 0 || D <= 0) return -1;
    if (dtype != 0 && dtype != 1) return -1;
    long double *w = malloc(sizeof(long double) * (size_t)S * S);
    if (!w) return -1;
    for (long bh = 0; bh < (long)B * H; ++bh) {
        const uint16_t *qh = q + (size_t)bh * S * D;
        const uint16_t *kh = k + (size_t)bh * S * D;
        const uint16_t *vh = v + (size_t)bh * S * D;
        for (int i = 0; i < S; ++i)
            for (int j = 0; j < S; ++j) {
                if (causal && j > i) { w[(size_t)i * S + j] = 0.0L; continue; }
                long double dot = 0.0L;
                for (int d = 0; d < D; ++d)
                    dot += (long double)widen(qh[(size_t)i * D + d], dtype) *
                           (long double)widen(kh[(size_t)j * D + d], dtype);
                w[(size_t)i * S + j] = expl((long double)scale * dot);
            }
        for (int i = 0; i < S; ++i) {
            long double z = 0.0L;
            for (int j = 0; j < S; ++j) z += w[(size_t)i * S + j];
            for (int j = 0; j < S; ++j)
                p[((size_t)bh * S + i) * S + j] = (double)(w[(size_t)i * S + j] / z);
            for (int d = 0; d < D; ++d) {
                long double acc = 0.0L;
                for (int j = 0; j < S; ++j)
                    acc += w[(size_t)i * S + j] * (long double)widen(vh[(size_t)j * D + d], dtype);
                o[((size_t)bh * S + i) * D + d] = (double)(acc / z);
            }
            lse[(size_t)bh * S + i] = (double)logl(z);
        }
    }
    free(w);
    return 0;
}

#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
