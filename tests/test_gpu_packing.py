"""Cost-aware packing on the GPU (paper Sec. 6.1, App. C.2): the latency model fitted to this
library's kernels predicts the time of packed micro-batches (packing is additive), and the Eq. 1
packing is no worse than fill-to-the-maximum first-fit-decreasing when both are run."""
import random

import pytest

pytestmark = pytest.mark.gpu


def test_balanced_packing_against_max_length_packing():
    import packing_study as ps
    rng = random.Random(4)
    # long-tailed draw (Sec. 3.1: short sequences dominate, long ones are rare), 4 x 32768 tokens
    lengths, cap = [], 4 * 32768
    while True:
        l = min(32768, max(64, int(512 * rng.random() ** (-1 / 1.1))))
        if sum(lengths) + l > cap:
            break
        lengths.append(l)
    res = ps.study(lengths, 32, 32, 128, 32768, 4, [512, 1024, 2048, 4096, 8192, 16384, 24576, 32768], reps=5,
                   warmup=2, node_limit=500_000)
    print(res)
    a, b, c = (res["model_ms"][k] for k in "abc")
    assert a > 0
    for l, err in zip(res["probe"]["lengths"], res["probe"]["fit_rel_err"]):
        assert err <= 0.15, (l, err)
    for name in ("max_length_ffd", "balanced_eq1"):
        for pred, meas in zip(res[name]["predicted_ms"], res[name]["measured_ms"]):
            assert abs(pred - meas) <= 0.20 * meas, (name, pred, meas)
    assert res["balanced_eq1"]["measured_objective_ms"] <= 1.03 * res["max_length_ffd"]["measured_objective_ms"]


def test_greedy_dispatch_against_length_buckets():
    import packing_study as ps
    rng = random.Random(8)
    lengths = []
    # an iteration without very long sequences: the case in which length buckets leave the
    # pipelines built for long sequences idle (Sec. 6.2)
    while sum(lengths) < 4 * 32768:
        lengths.append(min(12000, max(64, int(512 * rng.random() ** (-1 / 1.1)))))
    res = ps.dispatch_study(lengths, 32, 32, 128, [32768, 16384, 8192, 8192], [4, 4, 2, 2], 50,
                            [512, 1024, 2048, 4096, 8192, 16384, 24576, 32768], reps=5, warmup=2, seed=1)
    print(res)
    for name in ("length_buckets", "greedy_alg1"):
        for p in res[name]["pipelines"]:
            # Eq. 2 is a lower bound of the pipeline's time (up to the model's error)
            assert p["bound_ms"] <= 1.10 * p["measured_ms"] + 0.2, (name, p)
    assert res["greedy_alg1"]["max_measured_ms"] <= 1.03 * res["length_buckets"]["max_measured_ms"]
    assert res["greedy_alg1"]["max_bound_ms"] <= res["length_buckets"]["max_bound_ms"] * (1 + 1e-9)
