/*
 * hyd_plan.h - C ABI of the host-side planning steps that produce the packed buffers the
 * attention library (hyd_attn.h) consumes.  They are the part of Hydraulis (arXiv 2412.07894)
 * that sits directly upstream of the kernel: the latency model T(l) fitted to profiled times
 * (App. C.2), the packing of the sequences of one pipeline into micro-batches (Sec. 6.1, Eq. 1,
 * with the enumeration of the number of micro-batches V pruned as in App. D), and the greedy
 * dispatch of a mini-batch over pipelines (Sec. 6.2, Eq. 2; App. E, Alg. 1).
 *
 * Everything here is plain host arithmetic: all pointers are HOST pointers owned by the caller,
 * no HIP call is made, nothing is allocated that outlives a call, calls are re-entrant.
 * Errors are hyd_status codes (hyd_attn.h); outputs are untouched on error.
 */
#ifndef HYD_PLAN_H
#define HYD_PLAN_H

#include "hyd_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* T(l) = a l^2 + b l + c: time of one forward and backward over a sequence of l tokens (App. C.2:
 * the quadratic term is attention, the linear term everything else, the constant launch costs). */
typedef struct { double a, b, c; } hyd_latency_model;

/*
 * Least-squares fit of the model to n profiled points (App. C.2): minimises
 * sum_i w_i (T(l_i) - t_i)^2.
 *   lengths, times   n values each
 *   weights          n non-negative values, or NULL for w_i = 1 (the paper does not say how its
 *                    fit weighs the points; w_i = 1 / t_i^2 fits relative errors, which keeps
 *                    the short lengths from being drowned by the long ones)
 * HYD_ERR_SHAPE unless at least three distinct lengths carry a positive weight.
 */
hyd_status hyd_plan_fit_latency(const double* lengths, const double* times, const double* weights, int n,
                                hyd_latency_model* out);

/* T(l) of a model, evaluated as (a*l)*l + b*l + c. */
double hyd_plan_latency(const hyd_latency_model* model, double l);

/*
 * Packing of U sequences into exactly V micro-batches (Sec. 6.1, Eq. 1 with V given): minimise
 *     max_j ( sum of T(l_i) over the sequences of micro-batch j ) * (pp - 1 + V)
 * with every sequence in exactly one micro-batch and at most max_len tokens per micro-batch.
 * The packed time of a micro-batch is the sum of its sequences' times because attention does not
 * cross sequence boundaries (Sec. 6.1, "Solving for one V").
 *
 * Solved by depth-first branch and bound over the sequences in order of decreasing T, started
 * from a longest-processing-time-first packing.  The search visits at most node_limit nodes
 * (<= 0: 2,000,000); *proven_optimal is 1 when it finished (the returned packing then attains the
 * optimum of Eq. 1 for this V) and 0 when the limit cut it short (the best packing found so far
 * is returned).  *bound is a lower bound of the optimum: (pp-1+V) * max(largest T, sum T / V).
 *   assign           out, U entries: micro-batch (0..V-1) of every sequence
 * Errors: HYD_ERR_NULL; HYD_ERR_SHAPE (U < 0, V < 1, pp < 1, max_len < 1, a length < 1);
 * HYD_ERR_INFEASIBLE when no packing into V micro-batches respects max_len (proven, or none
 * found within the node limit).  U == 0 returns HYD_OK with objective 0.
 */
hyd_status hyd_plan_pack_fixed_v(const int32_t* lengths, int U, const hyd_latency_model* model,
                                 int64_t max_len, int V, int pp, int64_t node_limit,
                                 int32_t* assign, double* objective, double* bound, int* proven_optimal);

/*
 * The pruned range of V (App. D): from max(ceil(sum l / max_len), 1) to
 * min(floor(sum l / util_len), U), the upper end never below the lower one.  util_len is the
 * length from which a micro-batch uses the device well.
 */
hyd_status hyd_plan_v_range(const int32_t* lengths, int U, int64_t max_len, int64_t util_len,
                            int* v_lo, int* v_hi);

/*
 * Eq. 1 with V enumerated over hyd_plan_v_range: the best fixed-V packing, the smallest V on
 * ties.  node_limit applies to each V.  *proven_optimal is 1 only if every V of the range was
 * solved to the end.  Errors as above; HYD_ERR_INFEASIBLE when no V of the range admits a packing.
 */
hyd_status hyd_plan_pack(const int32_t* lengths, int U, const hyd_latency_model* model,
                         int64_t max_len, int64_t util_len, int pp, int64_t node_limit,
                         int32_t* assign, int* V, double* objective, int* proven_optimal);

/*
 * The packing the paper argues against (Sec. 3.1): fill micro-batches up to max_len, first fit
 * over the sequences in order of decreasing length (ties: lower index first).
 */
hyd_status hyd_plan_pack_ffd(const int32_t* lengths, int U, int64_t max_len, int32_t* assign, int* V);

/*
 * Greedy dispatch of B sequences over D pipelines (App. E, Alg. 1).  Pipelines are ordered by
 * non-increasing maximum length; sequence i may go to pipelines 0..J[i]-1.  In each trial the
 * sequences are visited in the order of the given permutation and each goes to the admissible
 * pipeline that minimises the largest running-time bound of Eq. 2,
 *     sum of T(l, P_j) over the pipeline's sequences + T(longest of them, P_j) * (pp_j - 1);
 * a candidate replaces the incumbent only when strictly better (lowest pipeline index and
 * earliest trial win ties).  The permutations are inputs: the random draws are the caller's.
 *   models, pps      D entries each
 *   perms            trials * B entries: trial t visits perms[t*B .. t*B+B-1], a permutation of 0..B-1
 *   assign           out, B entries: pipeline of every sequence
 *   cost             out: the largest Eq. 2 bound of the best trial
 * Errors: HYD_ERR_NULL; HYD_ERR_SHAPE (B < 0, D < 1, trials < 1, pp < 1, an entry of perms out of
 * range); HYD_ERR_INFEASIBLE when some J[i] < 1 (a sequence fits no pipeline) or J[i] > D.
 */
hyd_status hyd_plan_dispatch(const int32_t* lengths, int B, const int32_t* J,
                             const hyd_latency_model* models, const int32_t* pps, int D,
                             const int32_t* perms, int trials, int32_t* assign, double* cost);

#ifdef __cplusplus
}
#endif
#endif /* HYD_PLAN_H */
