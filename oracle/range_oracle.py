"""TEST INFRASTRUCTURE ONLY - plain fp64 reference for attention restricted to a range of queries
and a range of keys per sequence, and for the merge of partial results.  This is the arithmetic
of context parallelism, one of the three axes of the paper's parallel scheme <TP, PP, CP>
(arXiv 2412.07894, Sec. 2.1 on the parallel schemes; App. C.1 carries CP in the memory model):
each rank holds a chunk of the queries, the key/value chunks travel round a ring, every (query
chunk, key chunk) pair yields a partial output with its own log-sum-exp, and partials are merged
by the log-sum-exp rule.  The paper does not spell these formulas out; they follow from the
definition of softmax attention:

    keys of sequence s visible to its local row i in the call:  j in [kv_begin_s, kv_end_s), j <= i
    LSE_i  = ln sum_j exp(s_ij)  over those keys  (-inf when there is none),  O_i = softmax . V  (0)
    merge: LSE = ln(exp(LSE_a) + exp(LSE_b)),  O = exp(LSE_a - LSE) O_a + exp(LSE_b - LSE) O_b
    backward, with the FULL-row LSE and D_i = <dO_i, O_i> of the merged forward:
       P_ij = exp(s_ij - LSE_i),  dS_ij = P_ij (<dO_i, V_j> - D_i)
       dQ_i (rows of the query range) = scale sum_{j in key range} dS_ij K_j
       dK_j (keys of the key range)   = scale sum_{h in group} sum_{i in query range} dS_ij Q_i
       dV_j                           =       sum_{h in group} sum_{i in query range} P_ij dO_i

Dense numpy per (sequence, head), full score matrix with a boolean mask: no tiling, no running
statistics.  Only tests/ may import this module.
"""
import numpy as np


def _mask(L, qb, qe, kb, ke):
    i = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    return (j <= i) & (i >= qb) & (i < qe) & (j >= kb) & (j < ke)


def fwd_range(q, k, v, cu, scale, q_rng, kv_rng):
    """q [T,Hq,d], k, v [T,Hkv,d] float arrays; q_rng / kv_rng: per sequence (begin, end) in local
    positions.  Returns O [T,Hq,d] and LSE [Hq,T] (fp64); rows outside the query range are nan."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    T, hq, d = q.shape
    G = hq // k.shape[1]
    o = np.full((T, hq, d), np.nan)
    lse = np.full((hq, T), np.nan)
    for s in range(len(cu) - 1):
        r0, L = int(cu[s]), int(cu[s + 1] - cu[s])
        if L == 0:
            continue
        (qb, qe), (kb, ke) = q_rng[s], kv_rng[s]
        m = _mask(L, qb, qe, kb, ke)
        rows = np.arange(L)
        inq = (rows >= qb) & (rows < qe)
        for h in range(hq):
            g = h // G
            sc = scale * (q[r0:r0 + L, h] @ k[r0:r0 + L, g].T)
            sc = np.where(m, sc, -np.inf)
            mx = np.max(sc, axis=1)
            safe = np.where(np.isfinite(mx), mx, 0.0)
            e = np.exp(sc - safe[:, None])
            l = e.sum(axis=1)
            with np.errstate(divide="ignore", invalid="ignore"):
                p = np.where(l[:, None] > 0, e / l[:, None], 0.0)
                row_lse = np.where(l > 0, safe + np.log(l), -np.inf)
            out = p @ v[r0:r0 + L, g]
            o[r0:r0 + L, h][inq] = out[inq]
            lse[h, r0:r0 + L][inq] = row_lse[inq]
    return o, lse


def merge(o_a, lse_a, o_b, lse_b):
    """Log-sum-exp merge of two partial results (rows that are nan in both stay nan)."""
    lse_a = np.asarray(lse_a, dtype=np.float64); lse_b = np.asarray(lse_b, dtype=np.float64)
    with np.errstate(invalid="ignore", divide="ignore"):
        m = np.maximum(lse_a, lse_b)
        safe = np.where(np.isfinite(m), m, 0.0)
        wa, wb = np.exp(lse_a - safe), np.exp(lse_b - safe)
        tot = wa + wb
        lse = np.where(tot > 0, safe + np.log(tot), np.where(np.isnan(tot), np.nan, -np.inf))
        ca = np.where(tot > 0, wa / tot, 0.0)
        cb = np.where(tot > 0, wb / tot, 0.0)
    o = ca.T[:, :, None] * np.asarray(o_a, dtype=np.float64) + cb.T[:, :, None] * np.asarray(o_b, dtype=np.float64)
    return o, lse


def bwd_range(q, k, v, do, cu, scale, lse, dvec, q_rng, kv_rng):
    """Partial gradients of one (query range, key range) pair.  lse, dvec: [Hq,T] of the FULL rows.
    Returns dQ [T,Hq,d] (nan outside the query range), dK, dV [T,Hkv,d] (nan outside the key range)."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64); do = np.asarray(do, dtype=np.float64)
    T, hq, d = q.shape
    hkv = k.shape[1]
    G = hq // hkv
    dq = np.full((T, hq, d), np.nan)
    dk = np.full((T, hkv, d), np.nan)
    dv = np.full((T, hkv, d), np.nan)
    for s in range(len(cu) - 1):
        r0, L = int(cu[s]), int(cu[s + 1] - cu[s])
        if L == 0:
            continue
        (qb, qe), (kb, ke) = q_rng[s], kv_rng[s]
        m = _mask(L, qb, qe, kb, ke)
        rows = np.arange(L)
        inq = (rows >= qb) & (rows < qe)
        ink = (rows >= kb) & (rows < ke)
        dk[r0:r0 + L][ink] = 0.0
        dv[r0:r0 + L][ink] = 0.0
        for h in range(hq):
            g = h // G
            sc = scale * (q[r0:r0 + L, h] @ k[r0:r0 + L, g].T)
            p = np.where(m, np.exp(np.where(m, sc - lse[h, r0:r0 + L][:, None], 0.0)), 0.0)
            dp = do[r0:r0 + L, h] @ v[r0:r0 + L, g].T
            ds = p * (dp - dvec[h, r0:r0 + L][:, None])
            dq[r0:r0 + L, h][inq] = (scale * (ds @ k[r0:r0 + L, g]))[inq]
            dk[r0:r0 + L, g][ink] += (scale * (ds.T @ q[r0:r0 + L, h]))[ink]
            dv[r0:r0 + L, g][ink] += (p.T @ do[r0:r0 + L, h])[ink]
    return dq, dk, dv
