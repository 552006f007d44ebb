/* Calls every planning entry point of include/hyd_plan.h on small inputs, error paths included.
 * tests/test_plan_sanitize.py builds it as plain C (so the headers are checked as C too) together
 * with csrc/hyd_plan.cpp under -fsanitize=address,undefined; any report ends the run non-zero. */
#include <stdio.h>
#include <stdlib.h>

#include "hyd_plan.h"

int main(void) {
    int bad = 0;
    const double ls[] = {64, 128, 256, 512, 1024, 2048}, ts[6] = {0.11, 0.13, 0.18, 0.31, 0.70, 1.95};
    hyd_latency_model m;
    bad |= hyd_plan_fit_latency(ls, ts, NULL, 6, &m) != HYD_OK;
    bad |= hyd_plan_fit_latency(ls, ts, ts, 6, &m) != HYD_OK;
    bad |= hyd_plan_fit_latency(ls, ts, NULL, 2, &m) != HYD_ERR_SHAPE;
    const double t1k = hyd_plan_latency(&m, 1000.0);
    const int32_t lengths[] = {900, 40, 700, 512, 33, 2000, 64, 64, 1500, 300};
    const int U = 10;
    int32_t assign[10];
    double obj = 0, bound = 0, cost = 0;
    int proven = 0, V = 0, lo = 0, hi = 0;
    bad |= hyd_plan_pack_fixed_v(lengths, U, &m, 2048, 4, 4, 0, assign, &obj, &bound, &proven) != HYD_OK;
    bad |= hyd_plan_pack_fixed_v(lengths, U, &m, 2048, 2, 4, 0, assign, &obj, &bound, &proven) != HYD_ERR_INFEASIBLE;
    bad |= hyd_plan_pack_fixed_v(lengths, U, &m, 2048, 4, 4, 10, assign, &obj, &bound, &proven) > HYD_ERR_INFEASIBLE;
    bad |= hyd_plan_pack_fixed_v(lengths, 0, &m, 2048, 4, 4, 0, assign, &obj, &bound, &proven) != HYD_OK;
    bad |= hyd_plan_v_range(lengths, U, 2048, 512, &lo, &hi) != HYD_OK || lo < 1 || hi < lo;
    bad |= hyd_plan_pack(lengths, U, &m, 2048, 512, 4, 0, assign, &V, &obj, &proven) != HYD_OK;
    bad |= hyd_plan_pack(lengths, U, &m, 1000, 512, 4, 0, assign, &V, &obj, &proven) != HYD_ERR_INFEASIBLE;
    bad |= hyd_plan_pack_ffd(lengths, U, 2048, assign, &V) != HYD_OK;
    bad |= hyd_plan_pack_ffd(lengths, U, 100, assign, &V) != HYD_ERR_INFEASIBLE;
    const int32_t J[] = {2, 3, 2, 3, 3, 1, 3, 3, 1, 3}, pps[] = {4, 2, 1};
    const hyd_latency_model models[3] = {m, m, m};
    const int32_t perms[] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 9, 8, 7, 6, 5, 4, 3, 2, 1, 0};
    bad |= hyd_plan_dispatch(lengths, U, J, models, pps, 3, perms, 2, assign, &cost) != HYD_OK;
    const int32_t J_bad[] = {2, 3, 2, 3, 3, 0, 3, 3, 1, 3}, perm_bad[] = {0, 0, 2, 3, 4, 5, 6, 7, 8, 9};
    bad |= hyd_plan_dispatch(lengths, U, J_bad, models, pps, 3, perms, 2, assign, &cost) != HYD_ERR_INFEASIBLE;
    bad |= hyd_plan_dispatch(lengths, U, J, models, pps, 3, perm_bad, 1, assign, &cost) != HYD_ERR_SHAPE;
    bad |= hyd_plan_dispatch(lengths, 0, J, models, pps, 3, perms, 1, assign, &cost) != HYD_OK;
    printf("T(1000) %.4f V %d objective %.4f dispatch cost %.4f status %d\n", t1k, V, obj, cost, bad);
    return bad ? 1 : 0;
}
