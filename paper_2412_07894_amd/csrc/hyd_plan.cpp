// Host-side planning steps (include/hyd_plan.h): latency-model fit (paper App. C.2), packing of
// one pipeline's sequences into micro-batches (Sec. 6.1, Eq. 1; App. D), greedy dispatch over
// pipelines (Sec. 6.2, Eq. 2; App. E, Alg. 1).  Plain C++, no HIP.
#include "../../include/hyd_plan.h"

#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <limits>
#include <numeric>
#include <vector>

// every sum below is meant to round operation by operation (results are compared with a plain
// reference to the last bit where the order of operations is the same)
#pragma clang fp contract(off)

namespace {

inline double lat(const hyd_latency_model& m, double l) { return (m.a * l) * l + m.b * l + m.c; }

// ---- least squares by Householder QR on the design [x^2, x, 1], x = l / max l -----------------
bool fit3(const double* l, const double* t, const double* w, int n, hyd_latency_model* out) {
    double lmax = 0.0;
    for (int i = 0; i < n; ++i) lmax = std::max(lmax, fabs(l[i]));
    if (!(lmax > 0.0)) return false;
    std::vector<double> A(3 * (size_t)n), y(t, t + n);
    for (int i = 0; i < n; ++i) {
        const double x = l[i] / lmax;
        const double r = w ? sqrt(w[i]) : 1.0;            // weighted least squares: rows scaled by sqrt(w)
        A[0 * (size_t)n + i] = r * x * x;
        A[1 * (size_t)n + i] = r * x;
        A[2 * (size_t)n + i] = r;
        y[i] *= r;
    }
    double R[3][3] = {{0}};
    for (int k = 0; k < 3; ++k) {
        double* col = &A[k * (size_t)n];
        double norm = 0.0;
        for (int i = k; i < n; ++i) norm += col[i] * col[i];
        norm = sqrt(norm);
        if (!(norm > 1e-13)) return false;                 // rank deficient
        const double alpha = col[k] > 0 ? -norm : norm;
        std::vector<double> v(col + k, col + n);
        v[0] -= alpha;
        double vv = 0.0;
        for (double x : v) vv += x * x;
        if (!(vv > 0.0)) return false;
        auto reflect = [&](double* c) {
            double dot = 0.0;
            for (int i = k; i < n; ++i) dot += v[i - k] * c[i];
            const double f = 2.0 * dot / vv;
            for (int i = k; i < n; ++i) c[i] -= f * v[i - k];
        };
        for (int j = k; j < 3; ++j) reflect(&A[j * (size_t)n]);
        reflect(y.data());
        for (int j = k; j < 3; ++j) R[k][j] = A[j * (size_t)n + k];
    }
    if (fabs(R[2][2]) < 1e-12 * fabs(R[0][0])) return false;
    double c[3];
    for (int k = 2; k >= 0; --k) {
        double s = y[k];
        for (int j = k + 1; j < 3; ++j) s -= R[k][j] * c[j];
        c[k] = s / R[k][k];
    }
    out->a = c[0] / (lmax * lmax);
    out->b = c[1] / lmax;
    out->c = c[2];
    return true;
}

// ---- Eq. 1 with V given: branch and bound -----------------------------------------------------
struct PackSearch {
    int U, V;
    int64_t max_len, node_limit, nodes = 0;
    std::vector<double> t;            // T of the sequences, decreasing
    std::vector<int64_t> len;         // their lengths, same order
    std::vector<int64_t> suffix_len;  // total length of sequences k..U-1
    std::vector<int64_t> suffix_max;  // longest of sequences k..U-1
    std::vector<double> load;
    std::vector<int64_t> used;
    std::vector<int> cur, best;
    double best_max = std::numeric_limits<double>::infinity();
    double floor_max = 0.0;           // lower bound of the optimum's largest load
    bool stop = false;

    bool fits_rest(int k) const {     // necessary conditions for sequences k.. to fit at all
        int64_t room = 0, widest = 0;
        for (int j = 0; j < V; ++j) { room += max_len - used[j]; widest = std::max(widest, max_len - used[j]); }
        return suffix_len[k] <= room && suffix_max[k] <= widest;
    }
    void go(int k, double cur_max) {
        if (stop) return;
        if (k == U) {
            if (cur_max < best_max) {
                best_max = cur_max;
                best = cur;
                if (best_max <= floor_max * (1.0 + 1e-12)) stop = true;     // cannot be beaten
            }
            return;
        }
        if (++nodes > node_limit) { stop = true; return; }
        if (!fits_rest(k)) return;
        // candidate micro-batches, least loaded first; among micro-batches in the same state
        // (same load and fill) only the first is tried: the others give mirror images
        int order[64];
        std::vector<int> big;
        int* ord = order;
        if (V > 64) { big.resize(V); ord = big.data(); }
        for (int j = 0; j < V; ++j) ord[j] = j;
        std::sort(ord, ord + V, [&](int x, int y) { return load[x] != load[y] ? load[x] < load[y] : x < y; });
        for (int q = 0; q < V && !stop; ++q) {
            const int j = ord[q];
            if (used[j] + len[k] > max_len) continue;
            bool mirror = false;
            for (int r = 0; r < q; ++r)
                if (load[ord[r]] == load[j] && used[ord[r]] == used[j]) { mirror = true; break; }
            if (mirror) continue;
            const double before = load[j];
            const double nl = before + t[k];
            const double nm = std::max(cur_max, nl);
            if (nm >= best_max) continue;
            load[j] = nl; used[j] += len[k]; cur[k] = j;
            go(k + 1, nm);
            load[j] = before; used[j] -= len[k];
        }
    }
};

hyd_status pack_fixed_v(const int32_t* lengths, int U, const hyd_latency_model& m, int64_t max_len, int V,
                        int pp, int64_t node_limit, int32_t* assign, double* objective, double* bound,
                        int* proven) {
    if (U == 0) {
        *objective = 0.0; *bound = 0.0; *proven = 1;
        return HYD_OK;
    }
    int64_t total = 0;
    *proven = 1;
    for (int i = 0; i < U; ++i) {
        if (lengths[i] > max_len) return HYD_ERR_INFEASIBLE;
        total += lengths[i];
    }
    if (total > max_len * (int64_t)V) return HYD_ERR_INFEASIBLE;
    std::vector<int> idx(U);
    std::iota(idx.begin(), idx.end(), 0);
    std::vector<double> t_of(U);
    for (int i = 0; i < U; ++i) t_of[i] = lat(m, (double)lengths[i]);
    std::sort(idx.begin(), idx.end(), [&](int x, int y) {
        if (t_of[x] != t_of[y]) return t_of[x] > t_of[y];
        if (lengths[x] != lengths[y]) return lengths[x] > lengths[y];
        return x < y;
    });
    PackSearch s;
    s.U = U; s.V = V; s.max_len = max_len;
    s.node_limit = node_limit > 0 ? node_limit : 2000000;
    s.t.resize(U); s.len.resize(U);
    for (int k = 0; k < U; ++k) { s.t[k] = t_of[idx[k]]; s.len[k] = lengths[idx[k]]; }
    s.suffix_len.assign(U + 1, 0); s.suffix_max.assign(U + 1, 0);
    for (int k = U - 1; k >= 0; --k) {
        s.suffix_len[k] = s.suffix_len[k + 1] + s.len[k];
        s.suffix_max[k] = std::max(s.suffix_max[k + 1], s.len[k]);
    }
    double sum_t = 0.0, max_t = -std::numeric_limits<double>::infinity();
    for (int k = 0; k < U; ++k) { sum_t += s.t[k]; max_t = std::max(max_t, s.t[k]); }
    s.floor_max = std::max(max_t, sum_t / V);
    s.load.assign(V, 0.0); s.used.assign(V, 0); s.cur.assign(U, 0);
    // Start solution for tight capacities: first fit over the sequences by decreasing LENGTH (the
    // bin-packing heuristic), kept if it needs at most V micro-batches.  The first dive of the
    // search itself is the longest-processing-time-first packing (each sequence into the least
    // loaded micro-batch that has room), which is the better start when the cap is loose.
    {
        std::vector<int> by_len(U);
        std::iota(by_len.begin(), by_len.end(), 0);
        std::stable_sort(by_len.begin(), by_len.end(), [&](int x, int y) { return s.len[x] > s.len[y]; });
        std::vector<int64_t> room;
        std::vector<double> load;
        std::vector<int> a(U);
        bool ok = true;
        for (int k : by_len) {
            size_t j = 0;
            while (j < room.size() && room[j] < s.len[k]) ++j;
            if (j == room.size()) {
                if ((int)room.size() == V) { ok = false; break; }
                room.push_back(max_len); load.push_back(0.0);
            }
            room[j] -= s.len[k]; load[j] += s.t[k]; a[k] = (int)j;
        }
        if (ok) { s.best = a; s.best_max = *std::max_element(load.begin(), load.end()); }
    }
    s.go(0, -std::numeric_limits<double>::infinity());
    *proven = (s.nodes <= s.node_limit) ? 1 : 0;
    if (s.best.empty()) return HYD_ERR_INFEASIBLE;
    for (int k = 0; k < U; ++k) assign[idx[k]] = s.best[k];
    // objective recomputed in the order of the caller's sequences
    std::vector<double> load(V, 0.0);
    for (int i = 0; i < U; ++i) load[assign[i]] += t_of[i];
    *objective = *std::max_element(load.begin(), load.end()) * (double)(pp - 1 + V);
    *bound = s.floor_max * (double)(pp - 1 + V);
    return HYD_OK;
}

bool lengths_ok(const int32_t* lengths, int U) {
    for (int i = 0; i < U; ++i)
        if (lengths[i] < 1) return false;
    return true;
}

void v_range(const int32_t* lengths, int U, int64_t max_len, int64_t util_len, int* lo, int* hi) {
    int64_t total = 0;
    for (int i = 0; i < U; ++i) total += lengths[i];
    const int64_t l = std::max<int64_t>((total + max_len - 1) / max_len, 1);
    const int64_t h = std::max<int64_t>(std::min<int64_t>(total / util_len, U), l);
    *lo = (int)l;
    *hi = (int)h;
}

}  // namespace

extern "C" {

hyd_status hyd_plan_fit_latency(const double* lengths, const double* times, const double* weights, int n,
                                hyd_latency_model* out) {
    if (!lengths || !times || !out) return HYD_ERR_NULL;
    if (n < 3) return HYD_ERR_SHAPE;
    std::vector<double> u;
    for (int i = 0; i < n; ++i) {
        if (!std::isfinite(lengths[i]) || !std::isfinite(times[i])) return HYD_ERR_SHAPE;
        if (weights && !(weights[i] >= 0.0 && std::isfinite(weights[i]))) return HYD_ERR_SHAPE;
        if (!weights || weights[i] > 0.0) u.push_back(lengths[i]);
    }
    std::sort(u.begin(), u.end());
    if (std::unique(u.begin(), u.end()) - u.begin() < 3) return HYD_ERR_SHAPE;
    hyd_latency_model m;
    if (!fit3(lengths, times, weights, n, &m)) return HYD_ERR_SHAPE;
    *out = m;
    return HYD_OK;
}

double hyd_plan_latency(const hyd_latency_model* model, double l) {
    return model ? lat(*model, l) : 0.0;
}

hyd_status hyd_plan_pack_fixed_v(const int32_t* lengths, int U, const hyd_latency_model* model,
                                 int64_t max_len, int V, int pp, int64_t node_limit,
                                 int32_t* assign, double* objective, double* bound, int* proven_optimal) {
    if (!model || !objective || !bound || !proven_optimal || (U > 0 && (!lengths || !assign))) return HYD_ERR_NULL;
    if (U < 0 || V < 1 || pp < 1 || max_len < 1 || !lengths_ok(lengths, U)) return HYD_ERR_SHAPE;
    std::vector<int32_t> a(U);
    double obj = 0.0, bnd = 0.0;
    int proven = 0;
    const hyd_status st = pack_fixed_v(lengths, U, *model, max_len, V, pp, node_limit, a.data(), &obj, &bnd, &proven);
    if (st != HYD_OK) return st;
    std::copy(a.begin(), a.end(), assign);
    *objective = obj; *bound = bnd; *proven_optimal = proven;
    return HYD_OK;
}

hyd_status hyd_plan_v_range(const int32_t* lengths, int U, int64_t max_len, int64_t util_len,
                            int* v_lo, int* v_hi) {
    if (!v_lo || !v_hi || (U > 0 && !lengths)) return HYD_ERR_NULL;
    if (U < 0 || max_len < 1 || util_len < 1 || !lengths_ok(lengths, U)) return HYD_ERR_SHAPE;
    v_range(lengths, U, max_len, util_len, v_lo, v_hi);
    return HYD_OK;
}

hyd_status hyd_plan_pack(const int32_t* lengths, int U, const hyd_latency_model* model,
                         int64_t max_len, int64_t util_len, int pp, int64_t node_limit,
                         int32_t* assign, int* V, double* objective, int* proven_optimal) {
    if (!model || !V || !objective || !proven_optimal || (U > 0 && (!lengths || !assign))) return HYD_ERR_NULL;
    if (U < 0 || pp < 1 || max_len < 1 || util_len < 1 || !lengths_ok(lengths, U)) return HYD_ERR_SHAPE;
    int lo = 1, hi = 1;
    v_range(lengths, U, max_len, util_len, &lo, &hi);
    std::vector<int32_t> a(U), best_a;
    double best = std::numeric_limits<double>::infinity();
    int best_v = 0, all_proven = 1;
    double sum_t = 0.0, max_t = -std::numeric_limits<double>::infinity();
    for (int i = 0; i < U; ++i) {
        const double t = lat(*model, (double)lengths[i]);
        sum_t += t;
        max_t = std::max(max_t, t);
    }
    for (int v = lo; v <= hi; ++v) {
        // a V whose lower bound already reaches the best objective found cannot win (ties go to
        // the smaller V, which came first)
        if (U > 0 && std::max(max_t, sum_t / v) * (double)(pp - 1 + v) >= best) continue;
        double obj = 0.0, bnd = 0.0;
        int proven = 0;
        const hyd_status st = pack_fixed_v(lengths, U, *model, max_len, v, pp, node_limit, a.data(), &obj, &bnd, &proven);
        if (!proven) all_proven = 0;
        if (st == HYD_ERR_INFEASIBLE) continue;
        if (st != HYD_OK) return st;
        if (obj < best) { best = obj; best_v = v; best_a = a; }
    }
    if (best_v == 0) return HYD_ERR_INFEASIBLE;
    std::copy(best_a.begin(), best_a.end(), assign);
    *V = best_v; *objective = best; *proven_optimal = all_proven;
    return HYD_OK;
}

hyd_status hyd_plan_pack_ffd(const int32_t* lengths, int U, int64_t max_len, int32_t* assign, int* V) {
    if (!V || (U > 0 && (!lengths || !assign))) return HYD_ERR_NULL;
    if (U < 0 || max_len < 1 || !lengths_ok(lengths, U)) return HYD_ERR_SHAPE;
    for (int i = 0; i < U; ++i)
        if (lengths[i] > max_len) return HYD_ERR_INFEASIBLE;
    std::vector<int> idx(U);
    std::iota(idx.begin(), idx.end(), 0);
    std::stable_sort(idx.begin(), idx.end(), [&](int x, int y) { return lengths[x] > lengths[y]; });
    std::vector<int64_t> room;
    std::vector<int32_t> a(U);
    for (int i : idx) {
        size_t j = 0;
        while (j < room.size() && room[j] < lengths[i]) ++j;
        if (j == room.size()) room.push_back(max_len);
        room[j] -= lengths[i];
        a[i] = (int32_t)j;
    }
    std::copy(a.begin(), a.end(), assign);
    *V = (int)room.size();
    return HYD_OK;
}

hyd_status hyd_plan_dispatch(const int32_t* lengths, int B, const int32_t* J,
                             const hyd_latency_model* models, const int32_t* pps, int D,
                             const int32_t* perms, int trials, int32_t* assign, double* cost) {
    if (!models || !pps || !cost || (B > 0 && (!lengths || !J || !perms || !assign))) return HYD_ERR_NULL;
    if (B < 0 || D < 1 || trials < 1 || !lengths_ok(lengths, B)) return HYD_ERR_SHAPE;
    for (int j = 0; j < D; ++j)
        if (pps[j] < 1) return HYD_ERR_SHAPE;
    for (int i = 0; i < B; ++i)
        if (J[i] < 1 || J[i] > D) return HYD_ERR_INFEASIBLE;
    std::vector<char> seen(B);
    for (int tr = 0; tr < trials; ++tr) {
        std::fill(seen.begin(), seen.end(), 0);
        for (int k = 0; k < B; ++k) {
            const int i = perms[(size_t)tr * B + k];
            if (i < 0 || i >= B || seen[i]) return HYD_ERR_SHAPE;
            seen[i] = 1;
        }
    }
    const double inf = std::numeric_limits<double>::infinity();
    // Running state of one pipeline during a trial: the summed latency of its sequences, its
    // longest sequence, and the bound of Eq. 2 that follows from the two.
    struct Pipe {
        const hyd_latency_model* model;
        int stages;
        double sum;
        int64_t longest;
        double bound;
        double bound_with(int64_t l, double* sum_out, int64_t* longest_out) const {
            *longest_out = std::max(l, longest);
            *sum_out = sum + lat(*model, (double)l);
            return *sum_out + lat(*model, (double)*longest_out) * (double)(stages - 1);
        }
    };
    // The largest and the second largest bound, kept up to date as sequences are placed: the
    // "maximum over the other pipelines" that every candidate placement is compared with is one of
    // the two, so placing a sequence costs O(J_i) instead of O(J_i * D).
    struct TopTwo {
        double first, second;
        int first_at;
        void rebuild(const std::vector<Pipe>& ps) {
            first = second = -std::numeric_limits<double>::infinity();
            first_at = -1;
            for (int j = 0; j < (int)ps.size(); ++j) {
                if (ps[j].bound > first) { second = first; first = ps[j].bound; first_at = j; }
                else if (ps[j].bound > second) second = ps[j].bound;
            }
        }
        double without(int j) const { return j == first_at ? second : first; }
        // a bound that grows (the rule with monotone latency models) never needs a new runner-up
        void raise(int j, double b) {
            if (j == first_at) first = b;
            else if (b > first) { second = first; first = b; first_at = j; }
            else if (b > second) second = b;
        }
    };
    auto run_trial = [&](const int32_t* order, std::vector<Pipe>& pipes, std::vector<int32_t>& where) -> double {
        for (int j = 0; j < D; ++j) { pipes[j].sum = 0.0; pipes[j].longest = 0; pipes[j].bound = 0.0; }
        TopTwo top;
        top.rebuild(pipes);
        for (int k = 0; k < B; ++k) {
            const int i = order[k];
            double best = inf, best_sum = 0.0, best_bound = 0.0;
            int64_t best_longest = 0;
            int target = -1;
            for (int j = 0; j < J[i]; ++j) {               // admissible pipelines, first one wins a tie
                double sum_j;
                int64_t longest_j;
                const double bound_j = pipes[j].bound_with(lengths[i], &sum_j, &longest_j);
                const double overall = std::max(bound_j, top.without(j));
                if (overall < best) { best = overall; target = j; best_sum = sum_j; best_longest = longest_j; best_bound = bound_j; }
            }
            if (target < 0) return std::numeric_limits<double>::quiet_NaN();       // only with non-finite times
            where[i] = target;
            const bool grew = best_bound >= pipes[target].bound;
            pipes[target].sum = best_sum; pipes[target].longest = best_longest; pipes[target].bound = best_bound;
            if (grew) top.raise(target, best_bound);
            else top.rebuild(pipes);                       // a fitted model may price a sequence below zero
        }
        return B == 0 ? 0.0 : top.first;
    };
    std::vector<Pipe> pipes(D);
    for (int j = 0; j < D; ++j) { pipes[j].model = &models[j]; pipes[j].stages = pps[j]; }
    double best_cost = inf;
    std::vector<int32_t> best_assign(B), cur(B);
    for (int tr = 0; tr < trials; ++tr) {
        const double trial_cost = run_trial(perms + (size_t)tr * B, pipes, cur);
        if (trial_cost != trial_cost) return HYD_ERR_INFEASIBLE;
        if (trial_cost < best_cost) { best_cost = trial_cost; best_assign = cur; }
    }
    std::copy(best_assign.begin(), best_assign.end(), assign);
    *cost = best_cost;
    return HYD_OK;
}

}  // extern "C"
