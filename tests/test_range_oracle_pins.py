"""Pins of the range / merge reference (oracle/range_oracle.py): it must reduce to the pinned full
oracle when the ranges cover everything, and partial results over any partition of the keys or of
the queries must recombine into the full result (the identities context parallelism rests on).
CPU only."""
import numpy as np
import pytest

from oracle import attn_oracle as orc
from oracle import range_oracle as ro
from paper_2412_07894_amd import workloads as wl

LENGTHS = [5, 1, 12, 0, 9]
HQ, HKV, D = 4, 2, 8


@pytest.fixture(scope="module")
def case():
    cu, q, k, v, do = wl.custom(LENGTHS, HQ, HKV, D, "fp32", seed=3)
    scale = 0.3
    o, lse = orc.fwd(q, k, v, cu, scale)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, scale)
    dvec = np.einsum("thd,thd->ht", do.astype(np.float64), o)
    return dict(cu=cu, q=q, k=k, v=v, do=do, scale=scale, o=o, lse=lse, dq=dq, dk=dk, dv=dv, dvec=dvec)


def full(lengths):
    return [(0, L) for L in lengths]


def test_full_ranges_reduce_to_the_full_oracle(case):
    c = case
    o, lse = ro.fwd_range(c["q"], c["k"], c["v"], c["cu"], c["scale"], full(LENGTHS), full(LENGTHS))
    assert np.allclose(o, c["o"], rtol=0, atol=1e-12) and np.allclose(lse, c["lse"], rtol=0, atol=1e-12)
    dq, dk, dv = ro.bwd_range(c["q"], c["k"], c["v"], c["do"], c["cu"], c["scale"], c["lse"], c["dvec"],
                              full(LENGTHS), full(LENGTHS))
    for got, want in ((dq, c["dq"]), (dk, c["dk"]), (dv, c["dv"])):
        assert np.allclose(got, want, rtol=0, atol=1e-11)


@pytest.mark.parametrize("cuts", [(0.5,), (0.25, 0.75), (0.1, 0.2, 0.9)])
def test_key_chunks_merge_into_the_full_forward_and_sum_into_dq(case, cuts):
    c = case
    bounds = [[0] + [int(round(f * L)) for f in cuts] + [L] for L in LENGTHS]
    o_acc, lse_acc, dq_acc = None, None, 0.0
    dk_all = np.full_like(c["dk"], np.nan); dv_all = np.full_like(c["dv"], np.nan)
    for piece in range(len(cuts) + 1):
        kv = [(b[piece], b[piece + 1]) for b in bounds]
        o, lse = ro.fwd_range(c["q"], c["k"], c["v"], c["cu"], c["scale"], full(LENGTHS), kv)
        o_acc, lse_acc = (o, lse) if o_acc is None else ro.merge(o_acc, lse_acc, o, lse)
        dq, dk, dv = ro.bwd_range(c["q"], c["k"], c["v"], c["do"], c["cu"], c["scale"], c["lse"], c["dvec"],
                                  full(LENGTHS), kv)
        dq_acc = dq_acc + dq
        dk_all = np.where(np.isnan(dk), dk_all, dk); dv_all = np.where(np.isnan(dv), dv_all, dv)
    assert np.allclose(o_acc, c["o"], rtol=0, atol=1e-12)
    assert np.allclose(lse_acc, c["lse"], rtol=0, atol=1e-12)
    assert np.allclose(dq_acc, c["dq"], rtol=0, atol=1e-11)
    assert np.allclose(dk_all, c["dk"], rtol=0, atol=1e-11) and np.allclose(dv_all, c["dv"], rtol=0, atol=1e-11)


def test_query_chunks_partition_the_rows_and_sum_into_dk_dv(case):
    c = case
    halves = [[(0, L // 2) for L in LENGTHS], [(L // 2, L) for L in LENGTHS]]
    o_all = np.full_like(c["o"], np.nan); lse_all = np.full_like(c["lse"], np.nan)
    dq_all = np.full_like(c["dq"], np.nan); dk_acc, dv_acc = 0.0, 0.0
    for qr in halves:
        o, lse = ro.fwd_range(c["q"], c["k"], c["v"], c["cu"], c["scale"], qr, full(LENGTHS))
        o_all = np.where(np.isnan(o), o_all, o); lse_all = np.where(np.isnan(lse), lse_all, lse)
        dq, dk, dv = ro.bwd_range(c["q"], c["k"], c["v"], c["do"], c["cu"], c["scale"], c["lse"], c["dvec"],
                                  qr, full(LENGTHS))
        dq_all = np.where(np.isnan(dq), dq_all, dq)
        dk_acc = dk_acc + dk; dv_acc = dv_acc + dv
    assert np.allclose(o_all, c["o"], rtol=0, atol=1e-12) and np.allclose(lse_all, c["lse"], rtol=0, atol=1e-12)
    assert np.allclose(dq_all, c["dq"], rtol=0, atol=1e-11)
    assert np.allclose(dk_acc, c["dk"], rtol=0, atol=1e-11) and np.allclose(dv_acc, c["dv"], rtol=0, atol=1e-11)


def test_rows_that_see_no_key_of_the_range(case):
    c = case
    kv = [(L // 2, L) for L in LENGTHS]
    o, lse = ro.fwd_range(c["q"], c["k"], c["v"], c["cu"], c["scale"], full(LENGTHS), kv)
    for s, L in enumerate(LENGTHS):
        r0 = int(c["cu"][s])
        for i in range(L // 2):
            assert np.all(o[r0 + i] == 0.0) and np.all(np.isneginf(lse[:, r0 + i]))
        if L:
            i = L // 2                                    # first row with a key: sees exactly one
            assert np.allclose(o[r0 + i], c["v"][r0 + i].astype(np.float64).repeat(HQ // HKV, axis=0))


def test_merge_rules(case):
    c = case
    rng = np.random.default_rng(0)
    shp_o, shp_l = c["o"].shape, c["lse"].shape
    parts = [(rng.normal(size=shp_o), rng.normal(size=shp_l)) for _ in range(3)]
    ab = ro.merge(*parts[0], *parts[1]); ba = ro.merge(*parts[1], *parts[0])
    assert np.allclose(ab[0], ba[0]) and np.allclose(ab[1], ba[1])
    left = ro.merge(*ro.merge(*parts[0], *parts[1]), *parts[2])
    right = ro.merge(*parts[0], *ro.merge(*parts[1], *parts[2]))
    assert np.allclose(left[0], right[0]) and np.allclose(left[1], right[1])
    empty = (np.zeros(shp_o), np.full(shp_l, -np.inf))
    same = ro.merge(*parts[0], *empty)
    assert np.allclose(same[0], parts[0][0]) and np.allclose(same[1], parts[0][1])
    both = ro.merge(*empty, *empty)
    assert np.all(both[0] == 0.0) and np.all(np.isneginf(both[1]))
    # two-term closed form: equal LSEs average the outputs and add ln 2
    eq = ro.merge(parts[0][0], parts[0][1], parts[1][0], parts[0][1])
    assert np.allclose(eq[0], 0.5 * (parts[0][0] + parts[1][0])) and np.allclose(eq[1], parts[0][1] + np.log(2.0))
