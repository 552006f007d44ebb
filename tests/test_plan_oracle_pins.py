"""Pins of the planning oracle (oracle/plan_oracle.py) against things other than itself: values
worked by hand from the paper's formulas (Sec. 6.1 Eq. 1, Sec. 6.2 Eq. 2, App. C.2, App. D,
App. E Alg. 1), textbook special cases (number partitioning), exhaustive enumeration on tiny
inputs, and invariants.  CPU only."""
import itertools
import math
import random

import numpy as np
import pytest

from oracle import plan_oracle as po

LINEAR = (0.0, 1.0, 0.0)        # T(l) = l
SQUARE = (1.0, 0.0, 0.0)        # T(l) = l^2


def test_fit_recovers_an_exact_quadratic():
    a, b, c = 3.5e-7, 2.25e-3, 0.125
    l = np.array([128, 512, 1000, 4096, 20000, 32768], dtype=np.float64)
    got = po.fit_latency(l, a * l * l + b * l + c)
    assert np.allclose(got, (a, b, c), rtol=1e-8, atol=0)


def test_fit_through_three_points_is_the_interpolating_parabola():
    # Lagrange form evaluated at a fourth point
    l, t = [1.0, 2.0, 4.0], [2.0, 3.0, 11.0]
    m = po.fit_latency(l, t)
    x = 3.0
    lag = sum(t[i] * np.prod([(x - l[j]) / (l[i] - l[j]) for j in range(3) if j != i]) for i in range(3))
    assert abs(po.latency(m, x) - lag) < 1e-10
    for li, ti in zip(l, t):
        assert abs(po.latency(m, li) - ti) < 1e-10


def test_fit_residual_is_orthogonal_to_the_regressors():
    rng = np.random.default_rng(3)
    l = rng.uniform(100, 5000, size=40)
    t = 1e-6 * l * l + 1e-3 * l + 0.5 + rng.normal(0, 0.05, size=40)
    m = po.fit_latency(l, t)
    r = t - np.array([po.latency(m, x) for x in l])
    for reg in (l * l, l, np.ones_like(l)):
        assert abs(np.dot(r, reg)) <= 1e-7 * np.linalg.norm(reg) * np.linalg.norm(t)


def test_weighted_fit_properties():
    rng = np.random.default_rng(5)
    l = rng.uniform(100, 5000, size=30)
    t = 1e-6 * l * l + 1e-3 * l + 0.5 + rng.normal(0, 0.05, size=30)
    w = rng.uniform(0.1, 3.0, size=30)
    m = po.fit_latency(l, t, w)
    r = t - np.array([po.latency(m, x) for x in l])
    for reg in (l * l, l, np.ones_like(l)):              # weighted normal equations
        assert abs(np.dot(w * r, reg)) <= 1e-7 * np.linalg.norm(reg) * np.linalg.norm(t) * w.max()
    # integer weights are repetition counts
    k = np.array([1, 2, 3, 1, 2, 1])
    l6, t6 = l[:6], t[:6]
    rep = po.fit_latency(np.repeat(l6, k), np.repeat(t6, k))
    assert np.allclose(po.fit_latency(l6, t6, k.astype(float)), rep, rtol=1e-8)
    # equal weights change nothing
    assert np.allclose(po.fit_latency(l, t, np.full(30, 7.0)), po.fit_latency(l, t), rtol=1e-8)


def test_fit_needs_three_distinct_lengths():
    with pytest.raises(ValueError):
        po.fit_latency([1, 1, 2], [1, 1, 2])


def test_objective_worked_by_hand():
    # micro-batch loads 4 | 2+2 with T = l; Eq. 1: max load x (PP - 1 + V)
    assert po.packing_objective([4, 2, 2], [0, 1, 1], 2, LINEAR, pp=1) == 4 * 2
    assert po.packing_objective([4, 2, 2], [0, 1, 1], 2, LINEAR, pp=3) == 4 * 4
    assert po.packing_objective([4, 2, 2], [0, 0, 1], 2, SQUARE, pp=1) == (16 + 4) * 2
    # the constant term counts once per sequence, not once per micro-batch
    assert po.packing_objective([1, 1], [0, 0], 1, (0.0, 0.0, 7.0), pp=1) == 14.0


def test_number_partition_special_case():
    # T = l, no binding capacity: Eq. 1 with V fixed is multiway number partitioning
    lengths = [3, 1, 1, 2, 2, 1]
    for solver in (po.pack_fixed_v_bruteforce, po.pack_fixed_v_milp):
        obj2, a2 = solver(lengths, LINEAR, 100, 2, 1)
        obj3, a3 = solver(lengths, LINEAR, 100, 3, 1)
        assert obj2 == 5 * 2 and obj3 == 4 * 3
        assert po.check_packing(lengths, a2, 2, 100) and po.check_packing(lengths, a3, 3, 100)


def test_capacity_binds():
    lengths = [5, 5, 2, 2]
    for solver in (po.pack_fixed_v_bruteforce, po.pack_fixed_v_milp):
        obj, a = solver(lengths, SQUARE, 7, 2, 1)
        assert obj == (25 + 4) * 2 and po.check_packing(lengths, a, 2, 7)
        assert solver(lengths, SQUARE, 6, 2, 1) is None              # 5 + 2 > 6 and 5 + 5 > 6
        obj, a = solver(lengths, SQUARE, 6, 3, 1)
        assert obj == 25 * 3                                          # {5}, {5}, {2, 2}
        # a cap that forbids the balanced split costs something
        obj, a = solver([4, 4, 4, 4], SQUARE, 4, 4, 1)
        assert obj == 16 * 4


def test_single_micro_batch():
    lengths = [7, 9, 1]
    obj, a = po.pack_fixed_v_milp(lengths, (0.5, 2.0, 1.0), 17, 1, pp=4)
    want = sum(0.5 * l * l + 2.0 * l + 1.0 for l in lengths) * 4
    assert abs(obj - want) < 1e-9 and a == [0, 0, 0]
    assert po.pack_fixed_v_milp(lengths, SQUARE, 16, 1, pp=4) is None


@pytest.mark.parametrize("seed", range(12))
def test_milp_equals_enumeration_on_tiny_inputs(seed):
    rng = random.Random(seed)
    U = rng.randint(2, 7)
    V = rng.randint(1, 3)
    lengths = [rng.randint(1, 40) for _ in range(U)]
    model = (rng.uniform(0, 1e-2), rng.uniform(0, 1.0), rng.uniform(0, 2.0))
    max_len = max(max(lengths), int(sum(lengths) / V * rng.uniform(1.0, 1.6)))
    pp = rng.randint(1, 4)
    bf = po.pack_fixed_v_bruteforce(lengths, model, max_len, V, pp)
    mi = po.pack_fixed_v_milp(lengths, model, max_len, V, pp)
    assert (bf is None) == (mi is None)
    if bf is not None:
        assert abs(bf[0] - mi[0]) <= 1e-9 * bf[0]
        assert po.check_packing(lengths, mi[1], V, max_len)
        assert abs(po.packing_objective(lengths, mi[1], V, model, pp) - mi[0]) <= 1e-12 * mi[0]


def test_v_range_worked_by_hand():
    lengths = [5] * 20                                   # 100 tokens, 20 sequences
    assert po.v_range(lengths, 30, 12) == (4, 8)         # ceil(100/30), floor(100/12)
    assert po.v_range(lengths, 30, 4) == (4, 20)         # capped by the number of sequences
    assert po.v_range(lengths, 30, 1000) == (4, 4)       # never below the lower bound
    assert po.v_range(lengths, 1000, 1000) == (1, 1)


def test_enumeration_of_v():
    # equal sequences, PP = 1: V x max load is the same for every balanced V; the smallest V wins
    lengths = [8, 8, 8, 8]
    obj, V, a = po.pack(lengths, SQUARE, 32, 8, 1, solver=po.pack_fixed_v_bruteforce)
    assert (obj, V) == (4 * 64, 1)
    # a deep pipeline prefers more, smaller micro-batches: (PP-1+V) max load = (7+V) 256/V
    obj, V, a = po.pack(lengths, SQUARE, 32, 8, 8, solver=po.pack_fixed_v_bruteforce)
    assert V == 4 and obj == 64 * (7 + 4)
    # the enumeration is the minimum over the pruned range of the fixed-V optima
    lengths = [9, 7, 5, 4, 3, 1]
    lo, hi = po.v_range(lengths, 12, 5)
    each = [po.pack_fixed_v_bruteforce(lengths, SQUARE, 12, v, 3) for v in range(lo, hi + 1)]
    obj, V, a = po.pack(lengths, SQUARE, 12, 5, 3, solver=po.pack_fixed_v_bruteforce)
    assert obj == min(e[0] for e in each if e is not None)
    assert po.check_packing(lengths, a, V, 12)


def test_first_fit_decreasing_worked_by_hand():
    V, a = po.pack_ffd([7, 5, 4, 3, 1], 10)              # 7|3 and 5|4|1
    assert V == 2 and a == [0, 1, 1, 0, 1]
    V, a = po.pack_ffd([6, 6, 6], 10)
    assert V == 3 and sorted(a) == [0, 1, 2]
    with pytest.raises(ValueError):
        po.pack_ffd([11], 10)


def test_lower_bound_worked_by_hand():
    # Eq. 2: sum of T + T(longest) x (PP - 1)
    assert po.lower_bound([0, 1], [3, 1], SQUARE, pp=3) == (9 + 1) + 9 * 2
    assert po.lower_bound([1], [3, 1], SQUARE, pp=1) == 1
    assert po.lower_bound([], [3, 1], SQUARE, pp=5) == 0.0


def test_admissible_pipelines():
    assert po.admissible([4, 10, 20, 32], [32, 16, 8]) == [3, 2, 1, 1]
    assert po.admissible([33], [32, 16, 8]) == [0]


def test_greedy_dispatch_worked_by_hand():
    # two identical pipelines, T = l, PP = 1, identity order: 5 -> P1; 3 -> P2 (max 5 < 8);
    # 2 -> P2 (5 | 5 beats 7 | 3)
    cost, a = po.dispatch_greedy([5, 3, 2], [2, 2, 2], [LINEAR, LINEAR], [1, 1], [[0, 1, 2]])
    assert cost == 5 and a == [0, 1, 1]
    # PP = 2 on the first pipeline adds T(longest) once: 5 -> P1 costs 10, P2 costs 5, so P2;
    # 3 -> P1 costs 3 + 3 = 6 (max 6), P2 costs 8, so P1; 2 -> P1: 5 + 3 = 8, P2: 7, so P2
    cost, a = po.dispatch_greedy([5, 3, 2], [2, 2, 2], [LINEAR, LINEAR], [2, 1], [[0, 1, 2]])
    assert a == [1, 0, 1] and cost == 7
    # a sequence that only the first pipeline admits goes there whatever the load
    cost, a = po.dispatch_greedy([9, 1, 1], [1, 2, 2], [LINEAR, LINEAR], [1, 1], [[1, 2, 0]])
    assert a[0] == 0
    # best of several trials, earliest on ties
    c1, _ = po.dispatch_greedy([5, 3, 2], [2, 2, 2], [LINEAR, LINEAR], [1, 1], [[2, 1, 0]])
    cb, _ = po.dispatch_greedy([5, 3, 2], [2, 2, 2], [LINEAR, LINEAR], [1, 1], [[2, 1, 0], [0, 1, 2]])
    assert cb == min(c1, 5)


@pytest.mark.parametrize("seed", range(10))
def test_greedy_dispatch_invariants(seed):
    rng = random.Random(100 + seed)
    B, D = rng.randint(1, 7), rng.randint(1, 3)
    max_lens = sorted((rng.choice([16, 32, 64]) for _ in range(D)), reverse=True)
    lengths = [rng.randint(1, max_lens[0]) for _ in range(B)]
    J = po.admissible(lengths, max_lens)
    models = [(rng.uniform(0, 1e-2), rng.uniform(0.1, 1.0), rng.uniform(0, 1.0)) for _ in range(D)]
    pps = [rng.randint(1, 4) for _ in range(D)]
    perms = [rng.sample(range(B), B) for _ in range(5)]
    cost, a = po.dispatch_greedy(lengths, J, models, pps, perms)
    assert all(0 <= a[i] < J[i] for i in range(B))
    # the reported cost is the largest Eq. 2 bound of the final membership
    bounds = [po.lower_bound([i for i in range(B) if a[i] == j], lengths, models[j], pps[j]) for j in range(D)]
    assert abs(cost - max(bounds)) <= 1e-12 * max(1.0, cost)
    # never better than the optimum of the dispatching problem, and equal to it for one pipeline
    opt, _ = po.dispatch_bruteforce(lengths, J, models, pps)
    assert cost >= opt - 1e-12 * max(1.0, opt)
    if D == 1:
        assert abs(cost - opt) <= 1e-12 * max(1.0, opt)
    # more trials never hurt
    cost_all, _ = po.dispatch_greedy(lengths, J, models, pps, perms + [list(p) for p in itertools.permutations(range(B))][:50])
    assert cost_all <= cost + 1e-15
