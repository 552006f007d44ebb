"""Pins of the fp64 oracle against things other than itself: a numpy full-matrix brute force,
closed forms, invariances and finite differences.  A dropped term, a wrong sign or index, or a
transposed operand in oracle/attn_oracle.c fails at least one of these."""
import numpy as np
import pytest

from oracle import attn_oracle as orc
from paper_2412_07894_amd import workloads as wl
import brute


def case(lengths, hq, hkv, d, seed, dtype="fp32"):
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, dtype, seed)
    return cu, q, k, v, do, 1.0 / np.sqrt(d)


@pytest.mark.parametrize("lengths,hq,hkv,d", [
    ([1], 1, 1, 1), ([2], 1, 1, 2), ([3, 5], 2, 1, 4), ([8, 1, 2], 4, 2, 2), ([5, 3, 8, 1], 2, 2, 4),
    ([1, 7, 64, 184], 2, 2, 64), ([33, 0, 17], 4, 1, 8),
])
def test_brute_force(lengths, hq, hkv, d):
    cu, q, k, v, do, sc = case(lengths, hq, hkv, d, seed=11)
    o, lse = orc.fwd(q, k, v, cu, sc)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, sc)
    bo, blse, bdq, bdk, bdv = brute.packed(q, k, v, cu, sc, do)
    for a, b in ((o, bo), (lse, blse), (dq, bdq), (dk, bdk), (dv, bdv)):
        assert np.max(np.abs(a - b)) <= 1e-12 * max(1.0, np.max(np.abs(b)))


def test_packed_equals_unpacked_and_no_cross_contamination():
    lengths = [5, 19, 1, 40]
    cu, q, k, v, do, sc = case(lengths, 4, 2, 8, seed=3)
    o, lse = orc.fwd(q, k, v, cu, sc)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, sc)
    for s, L in enumerate(lengths):
        a, b = cu[s], cu[s + 1]
        c1 = np.array([0, L], dtype=np.int32)
        o1, l1 = orc.fwd(q[a:b], k[a:b], v[a:b], c1, sc)
        g1 = orc.bwd(q[a:b], k[a:b], v[a:b], do[a:b], c1, sc)
        assert np.array_equal(o1, o[a:b]) and np.array_equal(l1, lse[:, a:b])
        assert np.array_equal(g1[0], dq[a:b]) and np.array_equal(g1[1], dk[a:b]) and np.array_equal(g1[2], dv[a:b])
    # perturbing sequence 1 leaves every other sequence bitwise unchanged
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[cu[1]:cu[2]] += 1.0; k2[cu[1]:cu[2]] *= -2.0; v2[cu[1]:cu[2]] += 3.0
    o2, lse2 = orc.fwd(q2, k2, v2, cu, sc)
    g2 = orc.bwd(q2, k2, v2, do, cu, sc)
    keep = np.r_[0:cu[1], cu[2]:cu[4]]
    assert np.array_equal(o2[keep], o[keep]) and np.array_equal(lse2[:, keep], lse[:, keep])
    assert np.array_equal(g2[0][keep], dq[keep]) and np.array_equal(g2[1][keep], dk[keep])
    assert not np.array_equal(o2[cu[1]:cu[2]], o[cu[1]:cu[2]])
    # permuting the order of the sequences permutes the outputs
    perm = [2, 0, 3, 1]
    idx = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in perm])
    cup = wl.cu_seqlens([lengths[s] for s in perm])
    op, lp = orc.fwd(q[idx], k[idx], v[idx], cup, sc)
    assert np.array_equal(op, o[idx]) and np.array_equal(lp, lse[:, idx])


def test_softmax_rows_sum_to_one_and_match_lse():
    cu, q, k, v, do, sc = case([9, 30], 2, 1, 16, seed=5)
    o, lse = orc.fwd(q, k, v, cu, sc)
    for tok in (0, 8, 9, 20, 38):
        for h in (0, 1):
            p = orc.probs(q, k, cu, sc, tok, h)
            assert abs(p.sum() - 1.0) < 1e-14
            s = int(np.searchsorted(cu, tok, side="right") - 1)
            sc_row = sc * (k[cu[s]:tok + 1, 0].astype(np.float64) @ q[tok, h].astype(np.float64))
            assert np.allclose(p, np.exp(sc_row - lse[h, tok]), rtol=1e-13, atol=0)
            assert np.allclose(o[tok, h], p @ v[cu[s]:tok + 1, 0].astype(np.float64), rtol=1e-13, atol=1e-15)


def test_length_one_and_first_rows():
    lengths = [1, 4, 1, 6]
    cu, q, k, v, do, sc = case(lengths, 4, 2, 8, seed=8)
    o, lse = orc.fwd(q, k, v, cu, sc)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, sc)
    for s, L in enumerate(lengths):
        t = cu[s]
        for h in range(4):
            g = h // 2
            assert np.array_equal(o[t, h], v[t, g].astype(np.float64))      # row 0: P = [1]
            assert abs(lse[h, t] - sc * float(q[t, h].astype(np.float64) @ k[t, g].astype(np.float64))) < 1e-14
        if L == 1:
            assert np.all(dq[t] == 0.0) and np.all(dk[t] == 0.0)
            for g in range(2):
                assert np.allclose(dv[t, g], do[t, 2 * g].astype(np.float64) + do[t, 2 * g + 1], rtol=1e-15)


def test_uniform_attention_closed_forms():
    lengths = [7, 12]
    cu, q, k, v, do, sc = case(lengths, 2, 2, 4, seed=2)
    # Q = 0: P_ij = 1/(i+1), O_i = running mean of V, LSE_i = ln(i+1)
    o, lse = orc.fwd(np.zeros_like(q), k, v, cu, sc)
    for s, L in enumerate(lengths):
        a = cu[s]
        for i in range(L):
            assert np.allclose(o[a + i], v[a:a + i + 1].astype(np.float64).mean(axis=0), rtol=1e-14, atol=1e-16)
            assert np.allclose(lse[:, a + i], np.log(i + 1.0), rtol=0, atol=1e-15)
    # all keys of a sequence identical: same P, LSE shifted by scale*<q_i, k>
    kc = k.copy()
    for s in range(2):
        kc[cu[s]:cu[s + 1]] = k[cu[s]]
    o2, lse2 = orc.fwd(q, kc, v, cu, sc)
    assert np.allclose(o2, o, rtol=1e-13, atol=1e-15)
    for s, L in enumerate(lengths):
        a = cu[s]
        for i in range(L):
            for h in range(2):
                want = np.log(i + 1.0) + sc * float(q[a + i, h].astype(np.float64) @ kc[a, h].astype(np.float64))
                assert abs(lse2[h, a + i] - want) < 1e-13
    # scale = 0 is uniform too
    o3, lse3 = orc.fwd(q, k, v, cu, 0.0)
    assert np.allclose(o3, o, rtol=1e-14, atol=1e-16)


def test_constant_v_gives_zero_dq_dk():
    cu, q, k, v, do, sc = case([6, 9], 2, 1, 8, seed=4)
    vc = v.copy()
    for s in range(2):
        vc[cu[s]:cu[s + 1]] = v[cu[s]]
    o, _ = orc.fwd(q, k, vc, cu, sc)
    for s in range(2):
        assert np.allclose(o[cu[s]:cu[s + 1]], vc[cu[s]].astype(np.float64)[None], rtol=1e-14, atol=1e-15)
    dq, dk, dv = orc.bwd(q, k, vc, do, cu, sc)
    assert np.max(np.abs(dq)) < 1e-13 and np.max(np.abs(dk)) < 1e-13
    # dV_j = sum_i P_ij dO_i sums over j to sum_i dO_i (rows of P sum to one)
    for s in range(2):
        a, b = cu[s], cu[s + 1]
        assert np.allclose(dv[a:b, 0].sum(axis=0), do[a:b].astype(np.float64).sum(axis=(0, 1)), rtol=1e-12)


def test_key_shift_invariance():
    # bf16-valued inputs, so that k + c is exact in the float32 the oracle's interface takes
    cu, q, k, v, do, sc = case([10, 5], 4, 2, 8, seed=6, dtype="bf16")
    c = np.float32(0.75) * np.ones(8, dtype=np.float32)
    o, lse = orc.fwd(q, k, v, cu, sc)
    o2, lse2 = orc.fwd(q, k + c, v, cu, sc)
    assert np.allclose(o2, o, rtol=1e-12, atol=1e-14)
    shift = sc * (q.astype(np.float64) @ c.astype(np.float64))          # [T, Hq]
    assert np.allclose(lse2, lse + shift.T, rtol=1e-13, atol=1e-13)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, sc)
    for s in range(2):                                                  # sum_j dK_j = 0
        assert np.max(np.abs(dk[cu[s]:cu[s + 1]].sum(axis=0))) < 1e-12


def test_causality():
    cu, q, k, v, do, sc = case([12], 2, 2, 4, seed=9)
    o, lse = orc.fwd(q, k, v, cu, sc)
    dq, _, _ = orc.bwd(q, k, v, do, cu, sc)
    q2, k2, v2, do2 = q.copy(), k.copy(), v.copy(), do.copy()
    q2[7:] += 1; k2[7:] -= 2; v2[7:] *= 3; do2[7:] += 1
    o2, lse2 = orc.fwd(q2, k2, v2, cu, sc)
    dq2, _, _ = orc.bwd(q2, k2, v2, do2, cu, sc)
    assert np.array_equal(o2[:7], o[:7]) and np.array_equal(lse2[:, :7], lse[:, :7])
    assert np.array_equal(dq2[:7], dq[:7])
    assert not np.array_equal(o2[7:], o[7:])


def test_gqa_equals_mha_with_replicated_kv():
    cu, q, k, v, do, sc = case([9, 14], 6, 2, 8, seed=10)
    kr, vr = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)
    o, lse = orc.fwd(q, k, v, cu, sc)
    om, lm = orc.fwd(q, kr, vr, cu, sc)
    assert np.array_equal(o, om) and np.array_equal(lse, lm)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, sc)
    dqm, dkm, dvm = orc.bwd(q, kr, vr, do, cu, sc)
    assert np.array_equal(dq, dqm)
    assert np.allclose(dk, dkm.reshape(-1, 2, 3, 8).sum(axis=2), rtol=1e-13, atol=1e-14)
    assert np.allclose(dv, dvm.reshape(-1, 2, 3, 8).sum(axis=2), rtol=1e-13, atol=1e-14)


def test_finite_differences():
    """Central differences of the scalar <O, dO> with respect to every input element, with the
    forward taken from the BRUTE FORCE so that the gradient is pinned to a different forward."""
    lengths = [3, 5]
    cu, q, k, v, do, sc = case(lengths, 2, 1, 3, seed=12)
    q, k, v, do = (x.astype(np.float64) for x in (q, k, v, do))
    dq, dk, dv = orc.bwd(q, k, v, do, cu, sc)

    def loss(q_, k_, v_):
        o, _ = brute.packed(q_, k_, v_, cu, sc)
        return float((o * do).sum())

    eps = 1e-3      # inputs are float32 in the oracle's interface, so steps must survive the cast
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps; xm[idx] -= eps
            args_p = {"q": q, "k": k, "v": v}; args_m = dict(args_p)
            args_p[name] = xp; args_m[name] = xm
            num[idx] = (loss(args_p["q"], args_p["k"], args_p["v"]) - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * eps)
        assert np.max(np.abs(num - g)) <= 2e-6 * max(1.0, np.max(np.abs(g))), name


def test_linearity_in_v_and_do():
    cu, q, k, v, do, sc = case([11, 4], 2, 2, 8, seed=13)
    o, lse = orc.fwd(q, k, v, cu, sc)
    o2, lse2 = orc.fwd(q, k, 2.0 * v, cu, sc)
    assert np.allclose(o2, 2.0 * o, rtol=1e-15) and np.array_equal(lse2, lse)
    g = orc.bwd(q, k, v, do, cu, sc)
    g2 = orc.bwd(q, k, v, -4.0 * do, cu, sc)
    for a, b in zip(g, g2):
        assert np.allclose(b, -4.0 * a, rtol=1e-13, atol=1e-15)


def test_backward_given_stored_forward_results():
    """hyd_oracle_bwd_given (the backward as a function of the stored O and LSE it is handed)."""
    cu, q, k, v, do, sc = case([5, 1, 12, 0, 33], 4, 2, 8, seed=23)
    o, lse = orc.fwd(q, k, v, cu, sc)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, sc)
    # (1) on the exact O and LSE it is the plain backward (float32 copies: 6e-8 relative)
    for a, b in zip(orc.bwd_given(q, k, v, do, o, lse, cu, sc), (dq, dk, dv)):
        assert np.max(np.abs(a - b)) <= 2e-6 * max(1.0, np.max(np.abs(b)))
    # (2) perturbed O and LSE against the matrix form in numpy
    rng = np.random.default_rng(3)
    o_p = (o + 0.05 * rng.standard_normal(o.shape)).astype(np.float32)
    lse_p = (lse + 0.1 * rng.standard_normal(lse.shape)).astype(np.float32)
    got = orc.bwd_given(q, k, v, do, o_p, lse_p, cu, sc)
    for a, b in zip(got, brute.packed_given(q, k, v, cu, sc, do, o_p, lse_p)):
        assert np.max(np.abs(a - b)) <= 1e-12 * max(1.0, np.max(np.abs(b)))
    # (3) closed forms.  LSE + c for all rows: every P, hence every gradient, times exp(-c)
    c = 0.25
    lse32 = lse.astype(np.float32)
    base = orc.bwd_given(q, k, v, do, o_p, lse32, cu, sc)
    shifted = orc.bwd_given(q, k, v, do, o_p, lse32 + np.float32(c), cu, sc)
    for a, b in zip(shifted, base):
        assert np.allclose(a, np.exp(-c) * b, rtol=1e-6, atol=1e-6)    # lse + c is rounded to float32 row by row
    # O + delta in one row i of head h moves D_i by <dO_i, delta> and with it
    # dQ_i by -scale <dO_i, delta> sum_j P_ij K_j = -scale <dO_i, delta> * (the attention output over K)
    exact = orc.bwd_given(q, k, v, do, o.astype(np.float32), lse32, cu, sc)
    i, h = int(cu[2]) + 7, 3
    delta = rng.standard_normal(o.shape[2]).astype(np.float32)
    o_d = o.astype(np.float32).copy()
    o_d[i, h] += delta
    moved = orc.bwd_given(q, k, v, do, o_d, lse32, cu, sc)
    d_exact = float(np.dot(do[i, h].astype(np.float64), (o_d[i, h].astype(np.float64) - o.astype(np.float32)[i, h].astype(np.float64))))
    ok_attn, _ = orc.fwd(q, k, k, cu, sc)                   # softmax(QK^T) K: V replaced by K
    want = -sc * d_exact * ok_attn[i, h]
    assert np.allclose(moved[0][i, h] - exact[0][i, h], want, rtol=1e-5, atol=1e-8)
    other = np.ones(o.shape[0], dtype=bool); other[i] = False
    assert np.array_equal(moved[0][other], exact[0][other]) and np.array_equal(moved[2], exact[2])   # dV does not depend on O


def test_sampled_rows_and_cols_agree_with_full():
    """The one-output-at-a-time entry points are the same definition; they are pinned to the
    brute force directly."""
    lengths = [20, 1, 37]
    cu, q, k, v, do, sc = case(lengths, 4, 2, 8, seed=14)
    bo, blse, bdq, bdk, bdv = brute.packed(q, k, v, cu, sc, do)
    tok = np.array([0, 5, 19, 20, 21, 40, 57], dtype=np.int32)
    head = np.array([0, 3, 1, 2, 0, 3, 1], dtype=np.int32)
    o, lse, dq = orc.rows(q, k, v, do, cu, sc, tok, head)
    for n in range(len(tok)):
        assert np.allclose(o[n], bo[tok[n], head[n]], rtol=1e-12, atol=1e-14)
        assert abs(lse[n] - blse[head[n], tok[n]]) < 1e-12
        assert np.allclose(dq[n], bdq[tok[n], head[n]], rtol=1e-11, atol=1e-13)
    for s, g, cols in ((0, 0, [0, 7, 19]), (2, 1, [36, 3]), (1, 1, [0])):
        dk, dv = orc.cols(q, k, v, do, cu, sc, s, g, np.array(cols, dtype=np.int32))
        for n, j in enumerate(cols):
            assert np.allclose(dk[n], bdk[cu[s] + j, g], rtol=1e-11, atol=1e-13)
            assert np.allclose(dv[n], bdv[cu[s] + j, g], rtol=1e-11, atol=1e-13)


def test_argument_errors():
    cu, q, k, v, do, sc = case([4], 2, 1, 4, seed=1)
    with pytest.raises(ValueError):
        orc.fwd(q, k, v, np.array([0, 3], dtype=np.int32), sc)      # does not end at T
    with pytest.raises(ValueError):
        orc.fwd(q, k, v, np.array([1, 4], dtype=np.int32), sc)      # does not start at 0
    with pytest.raises(ValueError):
        orc.fwd(q[:, :1].repeat(3, axis=1), k.repeat(2, axis=1), v.repeat(2, axis=1), cu, sc)   # 3 % 2
