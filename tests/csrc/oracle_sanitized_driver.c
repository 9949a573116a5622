/*
 * Driver for a build of oracle/attn_oracle.c under AddressSanitizer and UndefinedBehaviorSanitizer (host only).
 * It runs the cases that touch every buffer of the oracle: the brute-force twin against the two-pass routine
 * on tiny shapes, a row subset against the full result, the degenerate S = 1, and the argument errors.
 * Prints "sanitized oracle ok" and returns 0, or says what differed and returns 1; a sanitizer finding aborts.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int attn_oracle_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int H, int S, int D, int causal,
                     double scale, int dtype, const int *rows, int nrows, double *o, double *lse);
int attn_oracle(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int H, int S, int D, int causal,
                double scale, int dtype, double *o, double *lse);
int attn_bruteforce(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int H, int S, int D, int causal,
                    double scale, int dtype, double *o, double *lse, double *p);

/* small finite 16-bit patterns: sign, an exponent near the bias, a few mantissa bits */
static uint32_t state = 12345u;
static uint16_t pattern(int dtype) {
    state = state * 1664525u + 1013904223u;
    const uint32_t r = state >> 8;
    const uint16_t sign = (uint16_t)((r & 1u) << 15);
    if (dtype == 0) return (uint16_t)(sign | ((13u + (r >> 1) % 4u) << 10) | ((r >> 4) & 0x3ffu));   /* binary16, |x| < 2 */
    return (uint16_t)(sign | ((125u + (r >> 1) % 4u) << 7) | ((r >> 4) & 0x7fu));                     /* bfloat16, |x| < 4 */
}

static int fail(const char *what, double got, double want) {
    printf("MISMATCH %s: got %.17g want %.17g\n", what, got, want);
    return 1;
}

static int one_case(int B, int H, int S, int D, int causal, int dtype) {
    const size_t n = (size_t)B * H * S * D, rowsn = (size_t)B * H * S;
    uint16_t *q = malloc(2 * n), *k = malloc(2 * n), *v = malloc(2 * n);
    double *o = malloc(8 * n), *lse = malloc(8 * rowsn), *ob = malloc(8 * n), *lb = malloc(8 * rowsn);
    double *p = malloc(8 * rowsn * S);
    if (!q || !k || !v || !o || !lse || !ob || !lb || !p) return fail("malloc", 0, 1);
    for (size_t i = 0; i < n; ++i) { q[i] = pattern(dtype); k[i] = pattern(dtype); v[i] = pattern(dtype); }
    const double scale = 1.0 / sqrt((double)D);
    int bad = 0;
    if (attn_oracle(q, k, v, B, H, S, D, causal, scale, dtype, o, lse) != 0) bad |= fail("attn_oracle rc", -1, 0);
    if (attn_bruteforce(q, k, v, B, H, S, D, causal, scale, dtype, ob, lb, p) != 0) bad |= fail("attn_bruteforce rc", -1, 0);
    for (size_t i = 0; i < n && !bad; ++i)
        if (fabs(o[i] - ob[i]) > 1e-12) bad |= fail("o against the brute-force twin", o[i], ob[i]);
    for (size_t i = 0; i < rowsn && !bad; ++i)
        if (fabs(lse[i] - lb[i]) > 1e-12) bad |= fail("lse against the brute-force twin", lse[i], lb[i]);
    for (size_t i = 0; i < rowsn && !bad; ++i) {   /* the weights of a row sum to 1, masked ones are 0 */
        double z = 0;
        for (int j = 0; j < S; ++j) {
            z += p[i * S + j];
            if (causal && j > (int)(i % S) && p[i * S + j] != 0.0) bad |= fail("masked weight", p[i * S + j], 0.0);
        }
        if (fabs(z - 1.0) > 1e-14) bad |= fail("row of weights", z, 1.0);
    }
    /* a row subset (first, last and one in between, not in order) is the same rows of the full result */
    int rows[3] = {S - 1, 0, S / 2};
    double *os = malloc(8 * (size_t)B * H * 3 * D), *ls = malloc(8 * (size_t)B * H * 3);
    if (!os || !ls) return fail("malloc", 0, 1);
    if (attn_oracle_rows(q, k, v, B, H, S, D, causal, scale, dtype, rows, 3, os, ls) != 0) bad |= fail("attn_oracle_rows rc", -1, 0);
    for (int bh = 0; bh < B * H && !bad; ++bh)
        for (int r = 0; r < 3; ++r) {
            for (int d = 0; d < D; ++d)
                if (os[((size_t)bh * 3 + r) * D + d] != o[((size_t)bh * S + rows[r]) * D + d])
                    bad |= fail("row subset o", os[((size_t)bh * 3 + r) * D + d], o[((size_t)bh * S + rows[r]) * D + d]);
            if (ls[(size_t)bh * 3 + r] != lse[(size_t)bh * S + rows[r]]) bad |= fail("row subset lse", ls[(size_t)bh * 3 + r], lse[(size_t)bh * S + rows[r]]);
        }
    /* argument errors touch nothing */
    int oob[1] = {S};
    if (attn_oracle_rows(q, k, v, B, H, S, D, causal, scale, dtype, oob, 1, os, ls) != -1) bad |= fail("row index out of range", 0, -1);
    if (attn_oracle_rows(NULL, k, v, B, H, S, D, causal, scale, dtype, rows, 3, os, ls) != -1) bad |= fail("null q", 0, -1);
    if (attn_oracle(q, k, v, B, H, 0, D, causal, scale, dtype, o, lse) != -1) bad |= fail("S = 0", 0, -1);
    if (attn_oracle(q, k, v, B, H, S, D, causal, scale, 2, o, lse) != -1) bad |= fail("dtype", 0, -1);
    if (attn_oracle_rows(q, k, v, B, H, S, D, causal, scale, dtype, rows, 0, os, ls) != 0) bad |= fail("empty row set", -1, 0);
    free(q); free(k); free(v); free(o); free(lse); free(ob); free(lb); free(p); free(os); free(ls);
    return bad;
}

int main(void) {
    int bad = 0;
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int causal = 0; causal < 2; ++causal) {
            bad |= one_case(2, 3, 9, 4, causal, dtype);
            bad |= one_case(1, 1, 1, 8, causal, dtype);      /* S = 1 */
            bad |= one_case(1, 5, 17, 3, causal, dtype);     /* more heads than threads may be, odd sizes */
        }
    if (!bad) printf("sanitized oracle ok\n");
    return bad;
}
