/*
 * fp64 CPU oracle for packed variable-length causal self-attention, forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or call this file;
 * it exists so that the GPU library can be compared with a slow, plain implementation of the
 * definition.  It shares no code with the HIP kernels.
 *
 * What it computes (paper Sec. 2.1, the paragraph on packing: packed sequences must not attend
 * to each other, so the mask is block diagonal and the cost is the sum of S_i^2 rather than
 * (sum S_i)^2; Sec. 6.1 "Solving for one V": a packed buffer costs the sum of its sequences;
 * Sec. 8.1: the models are decoder-only, hence causal).  For every sequence s occupying packed
 * rows [cu[s], cu[s+1]), every query head h (KV head g = h / (Hq/Hkv)) and every local row i:
 *
 *     s_ij   = scale * <Q_i, K_j>                  for 0 <= j <= i only
 *     m_i    = max_j s_ij,  l_i = sum_j exp(s_ij - m_i)
 *     P_ij   = exp(s_ij - m_i) / l_i,   LSE_i = m_i + ln l_i
 *     O_i    = sum_j P_ij V_j
 *
 * and, for an upstream gradient dO of O (the loss does not depend on LSE):
 *
 *     dP_ij  = <dO_i, V_j>,  D_i = sum_j P_ij dP_ij,  dS_ij = P_ij (dP_ij - D_i)
 *     dQ_i   = scale * sum_{j<=i} dS_ij K_j
 *     dK_j   = scale * sum_{h in group} sum_{i>=j} dS_ij Q_i
 *     dV_j   =         sum_{h in group} sum_{i>=j} P_ij dO_i
 *
 * Every sequence is first copied out of the packed buffer into its own dense arrays and then
 * handed to a routine that knows nothing about packing.  Rows are processed one at a time with a
 * two-pass softmax (max, then sum); there is no tiling, no running maximum, no fusion.
 * Inputs are float (bf16 and fp32 values are exactly representable) and are widened to double
 * before any arithmetic; all results are double.
 *
 * Pins (tests/test_oracle_pins.py): full-matrix brute force in numpy, packed == unpacked,
 * softmax rows summing to one, length-1 sequences, uniform-attention closed forms, constant-V,
 * key-shift invariance, causality, GQA == MHA with replicated KV, finite differences,
 * linearity in V and dO; the backward given stored forward results: equal to the plain backward
 * on the exact O and LSE, brute force with perturbed O and LSE, closed forms of both perturbations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double dot(const double* a, const double* b, int d) {
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += a[c] * b[c];
    return acc;
}

/* Probabilities of row i of one sequence: p[0..i], and the row's log-sum-exp. */
static double softmax_row(const double* q_i, const double* k, int i, int d, double scale, double* p) {
    double m = -INFINITY;
    for (int j = 0; j <= i; ++j) {
        p[j] = scale * dot(q_i, k + (size_t)j * d, d);
        if (p[j] > m) m = p[j];
    }
    double l = 0.0;
    for (int j = 0; j <= i; ++j) { p[j] = exp(p[j] - m); l += p[j]; }
    for (int j = 0; j <= i; ++j) p[j] /= l;
    return m + log(l);
}

/* One sequence, one query head, dense arrays q,k,v[L][d]: o[L][d], lse[L]. */
static void attn_fwd_one(const double* q, const double* k, const double* v, int L, int d,
                         double scale, double* o, double* lse, double* p) {
    for (int i = 0; i < L; ++i) {
        lse[i] = softmax_row(q + (size_t)i * d, k, i, d, scale, p);
        double* o_i = o + (size_t)i * d;
        for (int c = 0; c < d; ++c) o_i[c] = 0.0;
        for (int j = 0; j <= i; ++j)
            for (int c = 0; c < d; ++c) o_i[c] += p[j] * v[(size_t)j * d + c];
    }
}

/* One sequence, one query head.  dq is overwritten; dk and dv are ADDED to (the caller sums the
 * query heads of one KV group into them).  p, ds: scratch of L doubles each. */
static void attn_bwd_one(const double* q, const double* k, const double* v, const double* d_o,
                         int L, int d, double scale, double* dq, double* dk, double* dv,
                         double* p, double* ds) {
    for (int i = 0; i < L; ++i) {
        const double* q_i = q + (size_t)i * d;
        const double* do_i = d_o + (size_t)i * d;
        softmax_row(q_i, k, i, d, scale, p);
        double D = 0.0;
        for (int j = 0; j <= i; ++j) { ds[j] = dot(do_i, v + (size_t)j * d, d); D += p[j] * ds[j]; }
        for (int j = 0; j <= i; ++j) ds[j] = p[j] * (ds[j] - D);
        double* dq_i = dq + (size_t)i * d;
        for (int c = 0; c < d; ++c) dq_i[c] = 0.0;
        for (int j = 0; j <= i; ++j) {
            for (int c = 0; c < d; ++c) {
                dq_i[c] += scale * ds[j] * k[(size_t)j * d + c];
                dk[(size_t)j * d + c] += scale * ds[j] * q_i[c];
                dv[(size_t)j * d + c] += p[j] * do_i[c];
            }
        }
    }
}

/* The backward as a function of what a backward CALL is given.  A training step runs the forward
 * first, stores O (in the storage format, e.g. rounded to bf16) and LSE, and hands both to the
 * backward (the paper's unit of work is one forward and one backward propagation over a buffer,
 * Sec. 6.1), which does not recompute them: with o_in, lse_in[L] as given,
 *     P_ij = exp(s_ij - lse_in_i),   D_i = <dO_i, o_in_i>,
 * and then dS, dQ, dK, dV exactly as in attn_bwd_one.  With the exact O and LSE this IS
 * attn_bwd_one (P_ij = exp(s_ij - LSE_i) and D_i = sum_j P_ij dP_ij = <dO_i, O_i>); with a rounded
 * O it tells how much of a difference to the definition is owed to that rounding alone, i.e. to
 * the interface and not to the arithmetic of the implementation under test. */
static void attn_bwd_one_given(const double* q, const double* k, const double* v, const double* d_o,
                               const double* o_in, const double* lse_in, int L, int d, double scale,
                               double* dq, double* dk, double* dv, double* p, double* ds) {
    for (int i = 0; i < L; ++i) {
        const double* q_i = q + (size_t)i * d;
        const double* do_i = d_o + (size_t)i * d;
        const double D = dot(do_i, o_in + (size_t)i * d, d);
        for (int j = 0; j <= i; ++j) {
            p[j] = exp(scale * dot(q_i, k + (size_t)j * d, d) - lse_in[i]);
            ds[j] = p[j] * (dot(do_i, v + (size_t)j * d, d) - D);
        }
        double* dq_i = dq + (size_t)i * d;
        for (int c = 0; c < d; ++c) dq_i[c] = 0.0;
        for (int j = 0; j <= i; ++j) {
            for (int c = 0; c < d; ++c) {
                dq_i[c] += scale * ds[j] * k[(size_t)j * d + c];
                dk[(size_t)j * d + c] += scale * ds[j] * q_i[c];
                dv[(size_t)j * d + c] += p[j] * do_i[c];
            }
        }
    }
}

/* Copy rows [row0,row0+L) of head h out of a packed float tensor x[T][H][d] into dense doubles. */
static void unpack(const float* x, int H, int d, int row0, int L, int h, double* out) {
    for (int i = 0; i < L; ++i)
        for (int c = 0; c < d; ++c)
            out[(size_t)i * d + c] = (double)x[((size_t)(row0 + i) * H + h) * d + c];
}

static int check_cu(const int32_t* cu, int nseq, int T) {
    if (nseq < 0 || T < 0 || cu[0] != 0 || cu[nseq] != T) return 0;
    for (int s = 0; s < nseq; ++s) if (cu[s + 1] < cu[s]) return 0;
    return 1;
}

/* Packed forward.  q[T][Hq][d], k,v[T][Hkv][d] float; o[T][Hq][d], lse[Hq][T] double.
 * Returns 0, or -1 on malformed arguments, -2 on allocation failure. */
int hyd_oracle_fwd(const float* q, const float* k, const float* v, const int32_t* cu, int nseq,
                   int T, int hq, int hkv, int d, double scale, double* o, double* lse) {
    if (hq <= 0 || hkv <= 0 || hq % hkv || d <= 0 || !check_cu(cu, nseq, T)) return -1;
    const int G = hq / hkv;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < nseq; ++s) {
        for (int h = 0; h < hq; ++h) {
            const int row0 = cu[s], L = cu[s + 1] - cu[s];
            if (L == 0) continue;
            double* buf = (double*)malloc(sizeof(double) * ((size_t)4 * L * d + 2 * (size_t)L));
            if (!buf) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            double *qs = buf, *ks = qs + (size_t)L * d, *vs = ks + (size_t)L * d,
                   *os = vs + (size_t)L * d, *ls = os + (size_t)L * d, *p = ls + L;
            unpack(q, hq, d, row0, L, h, qs);
            unpack(k, hkv, d, row0, L, h / G, ks);
            unpack(v, hkv, d, row0, L, h / G, vs);
            attn_fwd_one(qs, ks, vs, L, d, scale, os, ls, p);
            for (int i = 0; i < L; ++i) {
                memcpy(o + ((size_t)(row0 + i) * hq + h) * d, os + (size_t)i * d, sizeof(double) * d);
                lse[(size_t)h * T + row0 + i] = ls[i];
            }
            free(buf);
        }
    }
    return fail ? -2 : 0;
}

/* Packed backward.  d_o[T][Hq][d] float; dq[T][Hq][d], dk,dv[T][Hkv][d] double (overwritten). */
int hyd_oracle_bwd(const float* q, const float* k, const float* v, const float* d_o,
                   const int32_t* cu, int nseq, int T, int hq, int hkv, int d, double scale,
                   double* dq, double* dk, double* dv) {
    if (hq <= 0 || hkv <= 0 || hq % hkv || d <= 0 || !check_cu(cu, nseq, T)) return -1;
    const int G = hq / hkv;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < nseq; ++s) {
        for (int g = 0; g < hkv; ++g) {
            const int row0 = cu[s], L = cu[s + 1] - cu[s];
            if (L == 0) continue;
            const size_t n = (size_t)L * d;
            double* buf = (double*)malloc(sizeof(double) * (7 * n + 2 * (size_t)L));
            if (!buf) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            double *qs = buf, *ks = qs + n, *vs = ks + n, *dos = vs + n, *dqs = dos + n,
                   *dks = dqs + n, *dvs = dks + n, *p = dvs + n, *ds = p + L;
            unpack(k, hkv, d, row0, L, g, ks);
            unpack(v, hkv, d, row0, L, g, vs);
            for (size_t e = 0; e < n; ++e) { dks[e] = 0.0; dvs[e] = 0.0; }
            for (int h = g * G; h < (g + 1) * G; ++h) {
                unpack(q, hq, d, row0, L, h, qs);
                unpack(d_o, hq, d, row0, L, h, dos);
                attn_bwd_one(qs, ks, vs, dos, L, d, scale, dqs, dks, dvs, p, ds);
                for (int i = 0; i < L; ++i)
                    memcpy(dq + ((size_t)(row0 + i) * hq + h) * d, dqs + (size_t)i * d, sizeof(double) * d);
            }
            for (int i = 0; i < L; ++i) {
                memcpy(dk + ((size_t)(row0 + i) * hkv + g) * d, dks + (size_t)i * d, sizeof(double) * d);
                memcpy(dv + ((size_t)(row0 + i) * hkv + g) * d, dvs + (size_t)i * d, sizeof(double) * d);
            }
            free(buf);
        }
    }
    return fail ? -2 : 0;
}

/* Packed backward given the stored forward results o_in[T][Hq][d] and lse_in[Hq][T] (float, the
 * values the backward call receives); see attn_bwd_one_given.  Outputs as hyd_oracle_bwd. */
int hyd_oracle_bwd_given(const float* q, const float* k, const float* v, const float* d_o,
                         const float* o_in, const float* lse_in, const int32_t* cu, int nseq, int T,
                         int hq, int hkv, int d, double scale, double* dq, double* dk, double* dv) {
    if (hq <= 0 || hkv <= 0 || hq % hkv || d <= 0 || !check_cu(cu, nseq, T)) return -1;
    const int G = hq / hkv;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < nseq; ++s) {
        for (int g = 0; g < hkv; ++g) {
            const int row0 = cu[s], L = cu[s + 1] - cu[s];
            if (L == 0) continue;
            const size_t n = (size_t)L * d;
            double* buf = (double*)malloc(sizeof(double) * (8 * n + 3 * (size_t)L));
            if (!buf) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            double *qs = buf, *ks = qs + n, *vs = ks + n, *dos = vs + n, *os = dos + n, *dqs = os + n,
                   *dks = dqs + n, *dvs = dks + n, *p = dvs + n, *ds = p + L, *ls = ds + L;
            unpack(k, hkv, d, row0, L, g, ks);
            unpack(v, hkv, d, row0, L, g, vs);
            for (size_t e = 0; e < n; ++e) { dks[e] = 0.0; dvs[e] = 0.0; }
            for (int h = g * G; h < (g + 1) * G; ++h) {
                unpack(q, hq, d, row0, L, h, qs);
                unpack(d_o, hq, d, row0, L, h, dos);
                unpack(o_in, hq, d, row0, L, h, os);
                for (int i = 0; i < L; ++i) ls[i] = (double)lse_in[(size_t)h * T + row0 + i];
                attn_bwd_one_given(qs, ks, vs, dos, os, ls, L, d, scale, dqs, dks, dvs, p, ds);
                for (int i = 0; i < L; ++i)
                    memcpy(dq + ((size_t)(row0 + i) * hq + h) * d, dqs + (size_t)i * d, sizeof(double) * d);
            }
            for (int i = 0; i < L; ++i) {
                memcpy(dk + ((size_t)(row0 + i) * hkv + g) * d, dks + (size_t)i * d, sizeof(double) * d);
                memcpy(dv + ((size_t)(row0 + i) * hkv + g) * d, dvs + (size_t)i * d, sizeof(double) * d);
            }
            free(buf);
        }
    }
    return fail ? -2 : 0;
}

static int seq_of_token(const int32_t* cu, int nseq, int t) {
    for (int s = 0; s < nseq; ++s) if (t >= cu[s] && t < cu[s + 1]) return s;
    return -1;
}

/* Outputs one at a time, for buffers too large for the full oracle: for each sample n, the packed
 * row tok[n] and query head head[n] give o_rows[n][d], lse_rows[n] and, when d_o != NULL,
 * dq_rows[n][d].  Row i of a sequence depends only on rows 0..i of that sequence, so each sample
 * unpacks just that prefix and evaluates the definition for the single row. */
int hyd_oracle_rows(const float* q, const float* k, const float* v, const float* d_o,
                    const int32_t* cu, int nseq, int T, int hq, int hkv, int d, double scale,
                    const int32_t* tok, const int32_t* head, int nsamp,
                    double* o_rows, double* lse_rows, double* dq_rows) {
    if (hq <= 0 || hkv <= 0 || hq % hkv || d <= 0 || !check_cu(cu, nseq, T)) return -1;
    const int G = hq / hkv;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < nsamp; ++n) {
        const int s = seq_of_token(cu, nseq, tok[n]);
        if (s < 0 || head[n] < 0 || head[n] >= hq) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        const int row0 = cu[s], i = tok[n] - row0, L = i + 1, h = head[n];
        const size_t m = (size_t)L * d;
        double* buf = (double*)malloc(sizeof(double) * (2 * m + 2 * (size_t)d + 2 * (size_t)L));
        if (!buf) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
        double *ks = buf, *vs = ks + m, *qi = vs + m, *doi = qi + d, *p = doi + d, *ds = p + L;
        unpack(k, hkv, d, row0, L, h / G, ks);
        unpack(v, hkv, d, row0, L, h / G, vs);
        unpack(q, hq, d, row0 + i, 1, h, qi);
        lse_rows[n] = softmax_row(qi, ks, i, d, scale, p);
        double* o_i = o_rows + (size_t)n * d;
        for (int c = 0; c < d; ++c) o_i[c] = 0.0;
        for (int j = 0; j <= i; ++j)
            for (int c = 0; c < d; ++c) o_i[c] += p[j] * vs[(size_t)j * d + c];
        if (d_o) {
            unpack(d_o, hq, d, row0 + i, 1, h, doi);
            double D = 0.0;
            for (int j = 0; j <= i; ++j) { ds[j] = dot(doi, vs + (size_t)j * d, d); D += p[j] * ds[j]; }
            double* dq_i = dq_rows + (size_t)n * d;
            for (int c = 0; c < d; ++c) dq_i[c] = 0.0;
            for (int j = 0; j <= i; ++j)
                for (int c = 0; c < d; ++c)
                    dq_i[c] += scale * p[j] * (ds[j] - D) * ks[(size_t)j * d + c];
        }
        free(buf);
    }
    return fail ? -3 : 0;
}

/* dK and dV of selected key rows of ONE sequence and ONE KV head: cols[n] are local key indices
 * j of sequence s.  dk_cols, dv_cols[ncols][d] are overwritten.  Every query row i >= min(cols)
 * of every query head of the group is evaluated in full (its softmax needs all keys 0..i). */
int hyd_oracle_cols(const float* q, const float* k, const float* v, const float* d_o,
                    const int32_t* cu, int nseq, int T, int hq, int hkv, int d, double scale,
                    int s, int g, const int32_t* cols, int ncols, double* dk_cols, double* dv_cols) {
    if (hq <= 0 || hkv <= 0 || hq % hkv || d <= 0 || !check_cu(cu, nseq, T)) return -1;
    if (s < 0 || s >= nseq || g < 0 || g >= hkv) return -1;
    const int G = hq / hkv, row0 = cu[s], L = cu[s + 1] - cu[s];
    int jmin = L;
    for (int n = 0; n < ncols; ++n) {
        if (cols[n] < 0 || cols[n] >= L) return -1;
        if (cols[n] < jmin) jmin = cols[n];
    }
    const size_t m = (size_t)L * d;
    double* ks = (double*)malloc(sizeof(double) * 2 * m);
    if (!ks) return -2;
    double* vs = ks + m;
    unpack(k, hkv, d, row0, L, g, ks);
    unpack(v, hkv, d, row0, L, g, vs);
    for (size_t e = 0; e < (size_t)ncols * d; ++e) { dk_cols[e] = 0.0; dv_cols[e] = 0.0; }
    int fail = 0;
#pragma omp parallel
    {
        double* acc = (double*)calloc(2 * (size_t)ncols * d + 2 * (size_t)d + 2 * (size_t)L, sizeof(double));
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        } else {
            double *adk = acc, *adv = adk + (size_t)ncols * d, *qi = adv + (size_t)ncols * d,
                   *doi = qi + d, *p = doi + d, *ds = p + L;
#pragma omp for collapse(2) schedule(dynamic, 8)
            for (int h = g * G; h < (g + 1) * G; ++h) {
                for (int i = jmin; i < L; ++i) {
                    unpack(q, hq, d, row0 + i, 1, h, qi);
                    unpack(d_o, hq, d, row0 + i, 1, h, doi);
                    softmax_row(qi, ks, i, d, scale, p);
                    double D = 0.0;
                    for (int j = 0; j <= i; ++j) { ds[j] = dot(doi, vs + (size_t)j * d, d); D += p[j] * ds[j]; }
                    for (int n = 0; n < ncols; ++n) {
                        const int j = cols[n];
                        if (j > i) continue;
                        const double dsj = p[j] * (ds[j] - D);
                        for (int c = 0; c < d; ++c) {
                            adk[(size_t)n * d + c] += scale * dsj * qi[c];
                            adv[(size_t)n * d + c] += p[j] * doi[c];
                        }
                    }
                }
            }
#pragma omp critical
            for (size_t e = 0; e < (size_t)ncols * d; ++e) { dk_cols[e] += adk[e]; dv_cols[e] += adv[e]; }
            free(acc);
        }
    }
    free(ks);
    return fail ? -2 : 0;
}

/* Softmax probabilities of one packed row (for the rows-sum-to-one pin): p_out[0..i]. */
int hyd_oracle_probs(const float* q, const float* k, const int32_t* cu, int nseq, int T, int hq,
                     int hkv, int d, double scale, int tok, int h, double* p_out) {
    if (hq <= 0 || hkv <= 0 || hq % hkv || d <= 0 || !check_cu(cu, nseq, T)) return -1;
    const int s = seq_of_token(cu, nseq, tok);
    if (s < 0 || h < 0 || h >= hq) return -1;
    const int row0 = cu[s], i = tok - row0, L = i + 1;
    double* ks = (double*)malloc(sizeof(double) * ((size_t)L * d + d));
    if (!ks) return -2;
    double* qi = ks + (size_t)L * d;
    unpack(k, hkv, d, row0, L, h / (hq / hkv), ks);
    unpack(q, hq, d, row0 + i, 1, h, qi);
    softmax_row(qi, ks, i, d, scale, p_out);
    free(ks);
    return 0;
}

int hyd_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
