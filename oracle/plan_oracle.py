"""TEST INFRASTRUCTURE ONLY - plain reference for the planning steps that sit directly upstream of
the attention hot path in Hydraulis (arXiv 2412.07894): the latency model, the packing problem of
one pipeline and the greedy dispatcher.  Only tests/ and measurement scripts' baseline legs may
import this module; the product planner (include/hyd_plan.h) shares no code with it.

What follows the paper and where:
  latency model       T(l) = a l^2 + b l + c, coefficients by least squares over profiled
                      (length, time) points                                   (App. C.2)
  packing objective   max over micro-batches of the summed T of its sequences, times
                      (PP - 1 + V); every sequence in exactly one micro-batch; packed
                      length of a micro-batch at most MaxLen                  (Sec. 6.1, Eq. 1)
  enumeration of V    V from max(sum l / MaxLen, 1) to min(sum l / UtilLen, U) (App. D)
  lower bound         sum of T over a pipeline's sequences + T(longest) (PP-1) (Sec. 6.2, Eq. 2)
  greedy dispatcher   Alg. 1 of App. E: random order, each sequence goes to the admissible
                      pipeline that minimises the largest lower bound; best of the trials

Readings where the text is ambiguous or garbled:
  * In Eq. 1 the factor (PP - 1 + V) multiplies the maximum (App. E.1 splits the optimum into
    max(...) (PP-1) and max(...) V, which only makes sense that way).
  * The bounds of the V range are fractions in the paper; V is an integer, so the lower bound is
    rounded up and the upper bound down, and the upper bound is never below the lower one.
  * In Alg. 1 the longest length of a pipeline after adding sequence i is max(l_i, longest so far)
    (the listing's `l_j` can only mean `l_i`).
  * Ties: a candidate replaces the incumbent only when strictly better, so the lowest pipeline
    index and the earliest trial win.  The random permutations are inputs.
"""
import itertools
import math

import numpy as np


def fit_latency(lengths, times, weights=None):
    """(a, b, c) of T(l) = a l^2 + b l + c by least squares (App. C.2): minimises
    sum_i w_i (T(l_i) - t_i)^2, w_i = 1 when no weights are given."""
    l = np.asarray(lengths, dtype=np.float64)
    t = np.asarray(times, dtype=np.float64)
    w = np.ones_like(l) if weights is None else np.asarray(weights, dtype=np.float64)
    if np.unique(l[w > 0]).size < 3:
        raise ValueError("need at least three distinct lengths")
    r = np.sqrt(w)
    design = np.stack([l * l, l, np.ones_like(l)], axis=1) * r[:, None]
    coef, *_ = np.linalg.lstsq(design, t * r, rcond=None)
    return tuple(float(x) for x in coef)


def latency(model, l):
    a, b, c = model
    return a * float(l) * float(l) + b * float(l) + c


def packing_objective(lengths, assign, n_batches, model, pp):
    """Eq. 1 for a given assignment (assign[i] = micro-batch of sequence i)."""
    load = [0.0] * n_batches
    for l, j in zip(lengths, assign):
        load[j] += latency(model, l)
    return max(load) * (pp - 1 + n_batches)


def check_packing(lengths, assign, n_batches, max_len):
    """True iff every sequence sits in one of the V micro-batches and none exceeds MaxLen."""
    if len(assign) != len(lengths):
        return False
    tot = [0] * n_batches
    for l, j in zip(lengths, assign):
        if not 0 <= j < n_batches:
            return False
        tot[j] += int(l)
    return all(t <= max_len for t in tot)


def pack_fixed_v_bruteforce(lengths, model, max_len, n_batches, pp):
    """All V^U assignments (tiny inputs only).  Returns (objective, assignment) or None."""
    best = None
    for assign in itertools.product(range(n_batches), repeat=len(lengths)):
        if not check_packing(lengths, assign, n_batches, max_len):
            continue
        obj = packing_objective(lengths, assign, n_batches, model, pp)
        if best is None or obj < best[0]:
            best = (obj, list(assign))
    return best


def pack_fixed_v_milp(lengths, model, max_len, n_batches, pp):
    """Eq. 1 handed to a mixed-integer solver as written: binaries o[i][j], one continuous z,
    minimise z subject to sum_i o[i][j] T_i <= z, sum_j o[i][j] = 1, sum_i o[i][j] l_i <= MaxLen.
    Returns (objective, assignment) or None when infeasible."""
    from scipy.optimize import Bounds, LinearConstraint, milp
    U, V = len(lengths), n_batches
    t = np.array([latency(model, l) for l in lengths])
    scale = float(t.max()) if U else 1.0
    tn = t / scale                                  # well-conditioned rows; objective rescaled below
    n = U * V + 1
    cost = np.zeros(n)
    cost[-1] = 1.0
    rows, lo, hi = [], [], []
    for j in range(V):                              # load of micro-batch j minus z <= 0
        r = np.zeros(n)
        for i in range(U):
            r[i * V + j] = tn[i]
        r[-1] = -1.0
        rows.append(r); lo.append(-np.inf); hi.append(0.0)
    for i in range(U):                              # every sequence exactly once
        r = np.zeros(n)
        r[i * V:(i + 1) * V] = 1.0
        rows.append(r); lo.append(1.0); hi.append(1.0)
    for j in range(V):                              # packed length
        r = np.zeros(n)
        for i in range(U):
            r[i * V + j] = float(lengths[i])
        rows.append(r); lo.append(-np.inf); hi.append(float(max_len))
    integrality = np.ones(n)
    integrality[-1] = 0
    res = milp(cost, constraints=LinearConstraint(np.array(rows), lo, hi), integrality=integrality,
               bounds=Bounds(np.zeros(n), np.concatenate([np.ones(U * V), [np.inf]])),
               options={"mip_rel_gap": 0.0})
    if not res.success:
        return None
    assign = [int(np.argmax(res.x[i * V:(i + 1) * V])) for i in range(U)]
    return packing_objective(lengths, assign, V, model, pp), assign


def v_range(lengths, max_len, util_len):
    """Pruned range of the number of micro-batches (App. D), as integers."""
    total, U = int(sum(lengths)), len(lengths)
    lo = max(math.ceil(total / max_len), 1)
    hi = max(min(total // util_len, U), lo)
    return lo, hi


def pack(lengths, model, max_len, util_len, pp, solver=pack_fixed_v_milp):
    """Enumerates V over the pruned range and keeps the best Eq. 1 optimum (smallest V on ties).
    Returns (objective, V, assignment)."""
    lo, hi = v_range(lengths, max_len, util_len)
    best = None
    for V in range(lo, hi + 1):
        got = solver(lengths, model, max_len, V, pp)
        if got is not None and (best is None or got[0] < best[0]):
            best = (got[0], V, got[1])
    return best


def pack_ffd(lengths, max_len):
    """The baseline the paper argues against: fill micro-batches to the maximum length, first fit
    over the sequences in order of decreasing length.  Returns (V, assignment)."""
    order = sorted(range(len(lengths)), key=lambda i: (-int(lengths[i]), i))
    room, assign = [], [0] * len(lengths)
    for i in order:
        for j, r in enumerate(room):
            if lengths[i] <= r:
                room[j] -= int(lengths[i]); assign[i] = j
                break
        else:
            if lengths[i] > max_len:
                raise ValueError("sequence longer than MaxLen")
            room.append(max_len - int(lengths[i])); assign[i] = len(room) - 1
    return len(room), assign


def lower_bound(members, lengths, model, pp):
    """Eq. 2: running-time lower bound of one pipeline holding the sequences `members`."""
    if not members:
        return 0.0
    return sum(latency(model, lengths[i]) for i in members) + \
        latency(model, max(lengths[i] for i in members)) * (pp - 1)


def admissible(lengths, max_lens):
    """J_i of Sec. 6.2: pipelines are ordered by non-increasing MaxLen; sequence i may run on
    pipelines 1..J_i, the ones whose MaxLen is at least l_i."""
    assert all(max_lens[j] >= max_lens[j + 1] for j in range(len(max_lens) - 1))
    return [sum(1 for m in max_lens if m >= l) for l in lengths]


def dispatch_greedy(lengths, J, models, pps, perms):
    """Alg. 1.  models[j], pps[j]: latency model and pipeline depth of pipeline j; perms: one
    permutation of range(B) per trial.  Returns (best cost, pipeline of every sequence)."""
    B, D = len(lengths), len(models)
    best_cost, best_assign = math.inf, None
    for perm in perms:
        C = [0.0] * D
        E = [0.0] * D
        longest = [0] * D
        assign = [-1] * B
        for i in perm:
            o_min, j_star, keep = math.inf, -1, None
            for j in range(J[i]):
                l_max = max(int(lengths[i]), longest[j])
                c_new = C[j] + latency(models[j], lengths[i])
                e_new = latency(models[j], l_max) * (pps[j] - 1)
                o_max = c_new + e_new
                for k in range(D):
                    if k != j:
                        o_max = max(o_max, C[k] + E[k])
                if o_max < o_min:
                    o_min, j_star, keep = o_max, j, (c_new, e_new, l_max)
            if j_star < 0:
                raise ValueError("a sequence fits no pipeline")
            assign[i] = j_star
            C[j_star], E[j_star], longest[j_star] = keep
        cost = max(C[j] + E[j] for j in range(D))
        if cost < best_cost:
            best_cost, best_assign = cost, assign
    return best_cost, best_assign


def dispatch_bruteforce(lengths, J, models, pps):
    """Optimum of the dispatching problem of Sec. 6.2 (max over pipelines of Eq. 2) by
    enumeration (tiny inputs only)."""
    B, D = len(lengths), len(models)
    best = (math.inf, None)
    for assign in itertools.product(*[range(J[i]) for i in range(B)]):
        cost = max(lower_bound([i for i in range(B) if assign[i] == j], lengths, models[j], pps[j])
                   for j in range(D))
        if cost < best[0]:
            best = (cost, list(assign))
    return best
