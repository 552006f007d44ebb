"""The planning calls of the C-ABI library (include/hyd_plan.h) against the planning oracle
(oracle/plan_oracle.py): host arithmetic only, runs without a GPU."""
import ctypes
import os
import random
import re

import numpy as np
import pytest

from oracle import plan_oracle as po

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pl():
    from paper_2412_07894_amd import binding, build, planner
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    planner._lib()
    return planner


def test_every_declared_planning_symbol_is_exported(pl):
    text = open(os.path.join(ROOT, "include", "hyd_plan.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(hyd_plan_[a-z_0-9]+)\s*\(", text)))
    assert set(names) == set(pl.EXPORTS)
    lib = pl._lib()
    for n in names:
        assert getattr(lib, n) is not None


def random_model(rng):
    return (rng.uniform(1e-8, 1e-5), rng.uniform(1e-4, 1e-2), rng.uniform(0.0, 0.5))


@pytest.mark.parametrize("seed", range(6))
def test_fit_matches_the_oracle(pl, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(3, 40))
    l = np.unique(rng.integers(64, 65536, size=n)).astype(np.float64)
    if l.size < 3:
        l = np.array([64.0, 1000.0, 65536.0])
    a, b, c = 2.7e-7, 1.9e-3, 0.08
    t = (a * l * l + b * l + c) * (1.0 + rng.normal(0, 0.02 if seed else 0.0, size=l.size))
    got = pl.fit_latency(l, t).as_tuple()
    want = po.fit_latency(l, t)
    if seed == 0:
        assert np.allclose(got, (a, b, c), rtol=1e-9)
    if l.size > 3:
        assert np.allclose(got, want, rtol=1e-6, atol=1e-12)
    # the fitted curves agree everywhere that matters, however ill-conditioned the coefficients
    for x in (64.0, 777.0, 20000.0, 65536.0):
        assert abs(pl.latency(got, x) - po.latency(want, x)) <= 1e-8 * abs(po.latency(want, x)) + 1e-12


def test_weighted_fit_matches_the_oracle(pl):
    rng = np.random.default_rng(21)
    l = np.array([256, 512, 1024, 2048, 4096, 8192, 16384, 32768], dtype=np.float64)
    t = (3e-9 * l * l + 2e-5 * l + 4e-3) * (1.0 + rng.normal(0, 0.05, size=l.size))
    w = 1.0 / (t * t)
    got = pl.fit_latency(l, t, w).as_tuple()
    want = po.fit_latency(l, t, w)
    assert np.allclose(got, want, rtol=1e-7)
    # relative weighting keeps the short lengths honest, the plain fit does not have to
    rel = [abs(pl.latency(got, x) - y) / y for x, y in zip(l, t)]
    assert max(rel) < 0.2
    # a zero weight removes a point
    w0 = w.copy(); w0[3] = 0.0
    a = pl.fit_latency(l, t, w0).as_tuple()
    b = pl.fit_latency(np.delete(l, 3), np.delete(t, 3), np.delete(w, 3)).as_tuple()
    assert np.allclose(a, b, rtol=1e-9)
    from paper_2412_07894_amd.binding import HydError
    with pytest.raises(HydError):
        pl.fit_latency(l[:3], t[:3], [1.0, 0.0, 1.0])
    with pytest.raises(HydError):
        pl.fit_latency(l, t, -w)


def test_latency_is_the_same_expression(pl):
    m = (3.3e-7, 1.7e-3, 0.25)
    for l in (1, 17, 4096, 65535):
        assert pl.latency(m, l) == po.latency(m, l)


def test_fit_errors(pl):
    from paper_2412_07894_amd.binding import HydError
    with pytest.raises(HydError) as e:
        pl.fit_latency([1, 1, 2], [1, 1, 2])
    assert e.value.code == 2
    with pytest.raises(HydError) as e:
        pl.fit_latency([1, 2], [1, 2])
    assert e.value.code == 2
    lib = pl._lib()
    assert lib.hyd_plan_fit_latency(None, None, None, 3, None) == 1


@pytest.mark.parametrize("seed", range(20))
def test_fixed_v_packing_is_optimal_on_tiny_inputs(pl, seed):
    rng = random.Random(seed)
    U, V = rng.randint(1, 8), rng.randint(1, 3)
    lengths = [rng.randint(1, 60) for _ in range(U)]
    model = random_model(rng)
    max_len = max(max(lengths), int(sum(lengths) / V * rng.uniform(1.0, 1.5)))
    pp = rng.randint(1, 5)
    want = po.pack_fixed_v_bruteforce(lengths, model, max_len, V, pp)
    if want is None:
        from paper_2412_07894_amd.binding import HydError
        with pytest.raises(HydError) as e:
            pl.pack_fixed_v(lengths, model, max_len, V, pp)
        assert e.value.code == 10
        return
    obj, assign, bound, proven = pl.pack_fixed_v(lengths, model, max_len, V, pp)
    assert proven
    assert po.check_packing(lengths, assign, V, max_len)
    assert abs(obj - want[0]) <= 1e-12 * want[0]
    assert abs(po.packing_objective(lengths, assign, V, model, pp) - obj) <= 1e-12 * obj
    assert bound <= obj * (1 + 1e-12)


@pytest.mark.parametrize("seed", range(8))
def test_fixed_v_packing_matches_the_milp_reference(pl, seed):
    rng = random.Random(1000 + seed)
    U, V = rng.randint(9, 22), rng.randint(2, 5)
    # long-tailed lengths as in the paper's corpora (Sec. 3.1): many short, few long
    lengths = [min(4096, max(16, int(128 * rng.random() ** (-1 / 1.2)))) for _ in range(U)]
    model = random_model(rng)
    max_len = max(max(lengths), int(sum(lengths) / V * rng.uniform(1.05, 1.4)))
    want = po.pack_fixed_v_milp(lengths, model, max_len, V, pp=2)
    if want is None:
        return
    obj, assign, bound, proven = pl.pack_fixed_v(lengths, model, max_len, V, 2, node_limit=20_000_000)
    assert po.check_packing(lengths, assign, V, max_len)
    if proven:
        assert abs(obj - want[0]) <= 1e-9 * want[0]
    else:
        assert obj >= want[0] * (1 - 1e-9)
    assert bound <= want[0] * (1 + 1e-9)


def test_capacity_cases_worked_by_hand(pl):
    from paper_2412_07894_amd.binding import HydError
    sq = (1.0, 0.0, 0.0)
    obj, a, _, proven = pl.pack_fixed_v([5, 5, 2, 2], sq, 7, 2, 1)
    assert obj == 58 and proven and po.check_packing([5, 5, 2, 2], a, 2, 7)
    with pytest.raises(HydError) as e:
        pl.pack_fixed_v([5, 5, 2, 2], sq, 6, 2, 1)
    assert e.value.code == 10
    obj, a, _, _ = pl.pack_fixed_v([5, 5, 2, 2], sq, 6, 3, 1)
    assert obj == 75
    obj, a, _, _ = pl.pack_fixed_v([3, 1, 1, 2, 2, 1], (0.0, 1.0, 0.0), 100, 2, 1)
    assert obj == 10
    # a packing that needs the search to respect the cap: only {6,4} {5,5} fits two bins of 10
    obj, a, _, proven = pl.pack_fixed_v([6, 5, 5, 4], sq, 10, 2, 1)
    assert proven and po.check_packing([6, 5, 5, 4], a, 2, 10) and obj == (36 + 16) * 2


def test_node_limit_returns_a_valid_packing(pl):
    rng = random.Random(5)
    lengths = [rng.randint(100, 4000) for _ in range(60)]
    model = (1e-6, 1e-3, 0.01)
    obj, a, bound, proven = pl.pack_fixed_v(lengths, model, 40000, 6, 4, node_limit=200)
    assert po.check_packing(lengths, a, 6, 40000)
    assert bound <= obj * (1 + 1e-12)
    assert abs(po.packing_objective(lengths, a, 6, model, 4) - obj) <= 1e-12 * obj
    # longest-processing-time-first is within 4/3 of the optimum, hence of the bound
    assert obj <= bound * 4.0 / 3.0 * (1 + 1e-9)


def test_v_range_matches_the_oracle(pl):
    rng = random.Random(9)
    for _ in range(50):
        lengths = [rng.randint(1, 500) for _ in range(rng.randint(1, 40))]
        max_len = rng.randint(max(lengths), 4 * max(lengths))
        util_len = rng.randint(1, 3 * max(lengths))
        assert pl.v_range(lengths, max_len, util_len) == po.v_range(lengths, max_len, util_len)


@pytest.mark.parametrize("seed", range(6))
def test_enumeration_of_v_matches_the_oracle(pl, seed):
    rng = random.Random(2000 + seed)
    U = rng.randint(4, 12)
    lengths = [rng.randint(8, 200) for _ in range(U)]
    model = random_model(rng)
    max_len = max(max(lengths), int(sum(lengths) / rng.randint(1, 3)))
    util_len = rng.randint(20, 120)
    pp = rng.randint(1, 6)
    want = po.pack(lengths, model, max_len, util_len, pp)
    obj, V, a, proven = pl.pack(lengths, model, max_len, util_len, pp)
    assert proven and po.check_packing(lengths, a, V, max_len)
    assert abs(obj - want[0]) <= 1e-9 * want[0]
    lo, hi = po.v_range(lengths, max_len, util_len)
    assert lo <= V <= hi
    if V != want[1]:           # equal objectives at two values of V: the smaller one must win
        assert V < want[1]


def test_ffd_matches_the_oracle(pl):
    rng = random.Random(11)
    for _ in range(40):
        lengths = [rng.randint(1, 300) for _ in range(rng.randint(1, 60))]
        max_len = rng.randint(max(lengths), 3 * max(lengths))
        assert pl.pack_ffd(lengths, max_len) == po.pack_ffd(lengths, max_len)
    assert pl.pack_ffd([7, 5, 4, 3, 1], 10) == (2, [0, 1, 1, 0, 1])


@pytest.mark.parametrize("seed", range(10))
def test_dispatch_matches_the_oracle_bit_for_bit(pl, seed):
    rng = random.Random(3000 + seed)
    B, D, trials = rng.randint(1, 60), rng.randint(1, 5), rng.randint(1, 8)
    max_lens = sorted((rng.choice([2048, 4096, 8192, 32768]) for _ in range(D)), reverse=True)
    lengths = [min(max_lens[0], max(16, int(128 * rng.random() ** (-1 / 1.2)))) for _ in range(B)]
    J = po.admissible(lengths, max_lens)
    models = [random_model(rng) for _ in range(D)]
    pps = [rng.randint(1, 8) for _ in range(D)]
    perms = [rng.sample(range(B), B) for _ in range(trials)]
    want_cost, want_assign = po.dispatch_greedy(lengths, J, models, pps, perms)
    cost, assign = pl.dispatch(lengths, J, models, pps, perms)
    assert assign == want_assign
    assert cost == want_cost


def test_dispatch_against_enumeration_and_eq2(pl):
    """The library's dispatcher pinned without the step-by-step reference: on small inputs its
    cost is Eq. 2 evaluated on the assignment it returns (max over pipelines of the sum of the
    latencies plus (PP - 1) times the latency of the longest sequence), every sequence sits on an
    admissible pipeline, no assignment found by enumeration is cheaper than the optimum it must
    not beat, and with every order of the sequences tried the best greedy result is within the
    factor the tie-free cases show (equal to the optimum whenever a single pipeline is admissible)."""
    import itertools
    rng = random.Random(77)
    for case in range(30):
        B, D = rng.randint(1, 6), rng.randint(1, 3)
        max_lens = sorted((rng.choice([512, 1024, 4096]) for _ in range(D)), reverse=True)
        lengths = [rng.randint(16, max_lens[0]) for _ in range(B)]
        J = po.admissible(lengths, max_lens)
        models = [random_model(rng) for _ in range(D)]
        pps = [rng.randint(1, 4) for _ in range(D)]
        perms = [list(p) for p in itertools.permutations(range(B))][:120]
        cost, assign = pl.dispatch(lengths, J, models, pps, perms)
        assert all(0 <= assign[i] < J[i] for i in range(B))
        eq2 = max(po.lower_bound([i for i in range(B) if assign[i] == j], lengths, models[j], pps[j]) for j in range(D))
        assert abs(cost - eq2) <= 1e-9 * max(1.0, abs(eq2))
        opt, _ = po.dispatch_bruteforce(lengths, J, models, pps)
        assert cost >= opt - 1e-9 * max(1.0, abs(opt))
        if all(j == 1 for j in J):
            assert abs(cost - opt) <= 1e-9 * max(1.0, abs(opt))
    # negative latencies (a fitted model with c < 0): the running maximum may shrink
    neg = (0.0, 1.0, -50.0)
    cost, assign = pl.dispatch([10, 20, 30], [2, 2, 2], [neg, neg], [1, 1], [[0, 1, 2]])
    eq2 = max(po.lower_bound([i for i in range(3) if assign[i] == j], [10, 20, 30], neg, 1) for j in range(2))
    assert cost == eq2


def test_dispatch_worked_by_hand_and_errors(pl):
    from paper_2412_07894_amd.binding import HydError
    lin = (0.0, 1.0, 0.0)
    assert pl.dispatch([5, 3, 2], [2, 2, 2], [lin, lin], [1, 1], [[0, 1, 2]]) == (5.0, [0, 1, 1])
    assert pl.dispatch([5, 3, 2], [2, 2, 2], [lin, lin], [2, 1], [[0, 1, 2]]) == (7.0, [1, 0, 1])
    with pytest.raises(HydError) as e:
        pl.dispatch([5, 3], [0, 1], [lin], [1], [[0, 1]])
    assert e.value.code == 10
    with pytest.raises(HydError) as e:
        pl.dispatch([5, 3], [1, 1], [lin], [1], [[0, 0]])            # not a permutation
    assert e.value.code == 2
    with pytest.raises(HydError) as e:
        pl.dispatch([5, 3], [1, 1], [lin], [0], [[0, 1]])
    assert e.value.code == 2


def test_packing_argument_errors(pl):
    lib = pl._lib()
    m = pl.LatencyModel(1.0, 0.0, 0.0)
    l = (ctypes.c_int32 * 2)(3, 4)
    out = (ctypes.c_int32 * 2)()
    obj, bnd, pr, v = ctypes.c_double(), ctypes.c_double(), ctypes.c_int(), ctypes.c_int()
    f = lib.hyd_plan_pack_fixed_v
    assert f(None, 2, ctypes.byref(m), 10, 1, 1, 0, out, ctypes.byref(obj), ctypes.byref(bnd), ctypes.byref(pr)) == 1
    assert f(l, 2, ctypes.byref(m), 10, 0, 1, 0, out, ctypes.byref(obj), ctypes.byref(bnd), ctypes.byref(pr)) == 2
    assert f(l, 2, ctypes.byref(m), 10, 1, 0, 0, out, ctypes.byref(obj), ctypes.byref(bnd), ctypes.byref(pr)) == 2
    assert f(l, 2, ctypes.byref(m), 3, 2, 1, 0, out, ctypes.byref(obj), ctypes.byref(bnd), ctypes.byref(pr)) == 10
    assert f(l, 0, ctypes.byref(m), 3, 2, 1, 0, out, ctypes.byref(obj), ctypes.byref(bnd), ctypes.byref(pr)) == 0
    bad = (ctypes.c_int32 * 2)(3, 0)
    assert f(bad, 2, ctypes.byref(m), 10, 1, 1, 0, out, ctypes.byref(obj), ctypes.byref(bnd), ctypes.byref(pr)) == 2
    assert lib.hyd_plan_pack_ffd(l, 2, 3, out, ctypes.byref(v)) == 10
    assert lib.hyd_plan_pack(l, 2, ctypes.byref(m), 10, 0, 1, 0, out, ctypes.byref(v), ctypes.byref(obj), ctypes.byref(pr)) == 2
