/* Calls every entry point of oracle/attn_oracle.c on small ragged inputs.  Built by
 * tests/test_oracle_sanitize.py together with the oracle under -fsanitize=address,undefined:
 * an out-of-bounds access, a use after free, signed overflow or a misaligned access in the
 * oracle ends the run with a non-zero status.  Prints a checksum so that the calls stay live. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int hyd_oracle_fwd(const float*, const float*, const float*, const int32_t*, int, int, int, int, int, double, double*, double*);
int hyd_oracle_bwd(const float*, const float*, const float*, const float*, const int32_t*, int, int, int, int, int, double,
                   double*, double*, double*);
int hyd_oracle_bwd_given(const float*, const float*, const float*, const float*, const float*, const float*, const int32_t*,
                         int, int, int, int, int, double, double*, double*, double*);
int hyd_oracle_rows(const float*, const float*, const float*, const float*, const int32_t*, int, int, int, int, int, double,
                    const int32_t*, const int32_t*, int, double*, double*, double*);
int hyd_oracle_cols(const float*, const float*, const float*, const float*, const int32_t*, int, int, int, int, int, double,
                    int, int, const int32_t*, int, double*, double*);
int hyd_oracle_probs(const float*, const float*, const int32_t*, int, int, int, int, int, double, int, int, double*);
int hyd_oracle_threads(void);

static float* filled(size_t n, unsigned seed) {
    float* x = (float*)malloc(sizeof(float) * n);
    for (size_t i = 0; i < n; ++i) { seed = seed * 1664525u + 1013904223u; x[i] = (float)((int)(seed >> 20) - 2048) / 1024.0f; }
    return x;
}

int main(void) {
    const int32_t cu[] = {0, 1, 1, 8, 41, 44};           /* lengths 1, 0, 7, 33, 3 */
    const int nseq = 5, T = 44, hq = 4, hkv = 2, d = 8;
    const double scale = 0.35;
    float *q = filled((size_t)T * hq * d, 1), *k = filled((size_t)T * hkv * d, 2), *v = filled((size_t)T * hkv * d, 3),
          *dO = filled((size_t)T * hq * d, 4);
    double *o = malloc(sizeof(double) * T * hq * d), *lse = malloc(sizeof(double) * hq * T);
    double *dq = malloc(sizeof(double) * T * hq * d), *dk = malloc(sizeof(double) * T * hkv * d), *dv = malloc(sizeof(double) * T * hkv * d);
    int bad = 0;
    bad |= hyd_oracle_fwd(q, k, v, cu, nseq, T, hq, hkv, d, scale, o, lse);
    bad |= hyd_oracle_bwd(q, k, v, dO, cu, nseq, T, hq, hkv, d, scale, dq, dk, dv);
    double sum = dq[0] + dk[T * hkv * d - 1] + dv[5] + o[T * hq * d - 1] + lse[hq * T - 1];
    float *of = malloc(sizeof(float) * T * hq * d), *lf = malloc(sizeof(float) * hq * T);
    for (int i = 0; i < T * hq * d; ++i) of[i] = (float)o[i];
    for (int i = 0; i < hq * T; ++i) lf[i] = (float)lse[i];
    bad |= hyd_oracle_bwd_given(q, k, v, dO, of, lf, cu, nseq, T, hq, hkv, d, scale, dq, dk, dv);
    sum += dq[1] + dk[2] + dv[3];
    const int32_t tok[] = {0, 1, 7, 8, 40, 43}, head[] = {0, 3, 1, 2, 3, 0};
    double ro[6 * 8], rl[6], rq[6 * 8];
    bad |= hyd_oracle_rows(q, k, v, dO, cu, nseq, T, hq, hkv, d, scale, tok, head, 6, ro, rl, rq);
    bad |= hyd_oracle_rows(q, k, v, NULL, cu, nseq, T, hq, hkv, d, scale, tok, head, 6, ro, rl, rq);
    const int32_t cols[] = {0, 5, 32};
    double ck[3 * 8], cv[3 * 8];
    bad |= hyd_oracle_cols(q, k, v, dO, cu, nseq, T, hq, hkv, d, scale, 3, 1, cols, 3, ck, cv);
    double p[33];
    bad |= hyd_oracle_probs(q, k, cu, nseq, T, hq, hkv, d, scale, 40, 2, p);
    sum += ro[0] + rl[5] + rq[47] + ck[0] + cv[23] + p[32];
    /* argument errors must be reported, not crash */
    const int32_t bad_cu[] = {0, 5, 3, 44, 44, 44};
    if (hyd_oracle_fwd(q, k, v, bad_cu, nseq, T, hq, hkv, d, scale, o, lse) == 0) bad = 1;
    if (hyd_oracle_bwd(q, k, v, dO, cu, nseq, T, 3, 2, d, scale, dq, dk, dv) == 0) bad = 1;
    const int32_t far_col[] = {40};
    if (hyd_oracle_cols(q, k, v, dO, cu, nseq, T, hq, hkv, d, scale, 2, 0, far_col, 1, ck, cv) == 0) bad = 1;
    printf("threads %d checksum %.6f status %d\n", hyd_oracle_threads(), sum, bad);
    free(q); free(k); free(v); free(dO); free(o); free(lse); free(dq); free(dk); free(dv); free(of); free(lf);
    return bad ? 1 : 0;
}
