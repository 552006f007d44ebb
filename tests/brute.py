"""Full-matrix brute force for tiny inputs, used only to pin the oracle.  It materialises the
L x L score matrix of one sequence and one head with -inf above the diagonal, applies a generic
row softmax and generic matrix products, and takes gradients by the matrix formulas
  dV = P^T dO,  dP = dO V^T,  dS = P * (dP - rowsum(P * dP)),  dQ = scale dS K,  dK = scale dS^T Q.
It shares nothing with oracle/ (different language, different loop structure)."""
import numpy as np


def one_head(q, k, v, scale, d_o=None):
    L = q.shape[0]
    s = scale * (q.astype(np.float64) @ k.astype(np.float64).T)
    s[np.triu_indices(L, 1)] = -np.inf
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    p = e / l
    o = p @ v.astype(np.float64)
    lse = (m + np.log(l))[:, 0]
    if d_o is None:
        return o, lse, p
    d_o = d_o.astype(np.float64)
    dv = p.T @ d_o
    dp = d_o @ v.astype(np.float64).T
    ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
    dq = scale * ds @ k.astype(np.float64)
    dk = scale * ds.T @ q.astype(np.float64)
    return o, lse, p, dq, dk, dv


def packed(q, k, v, cu, scale, d_o=None):
    T, hq, d = q.shape
    hkv = k.shape[1]
    G = hq // hkv
    o = np.zeros((T, hq, d)); lse = np.zeros((hq, T))
    dq = np.zeros((T, hq, d)); dk = np.zeros((T, hkv, d)); dv = np.zeros((T, hkv, d))
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if a == b:
            continue
        for h in range(hq):
            g = h // G
            r = one_head(q[a:b, h], k[a:b, g], v[a:b, g], scale, None if d_o is None else d_o[a:b, h])
            o[a:b, h] = r[0]; lse[h, a:b] = r[1]
            if d_o is not None:
                dq[a:b, h] = r[3]; dk[a:b, g] += r[4]; dv[a:b, g] += r[5]
    return (o, lse) if d_o is None else (o, lse, dq, dk, dv)


def one_head_given(q, k, v, scale, d_o, o_in, lse_in):
    """Matrix form of the backward that takes the stored forward results as given:
    P = exp(S - lse_in) below and on the diagonal, D = rowsum(dO * o_in)."""
    L = q.shape[0]
    q, k, v, d_o = (x.astype(np.float64) for x in (q, k, v, d_o))
    p = np.tril(np.exp(scale * (q @ k.T) - np.asarray(lse_in, dtype=np.float64)[:, None]))
    ds = p * (d_o @ v.T - (d_o * np.asarray(o_in, dtype=np.float64)).sum(axis=1, keepdims=True))
    return scale * ds @ k, scale * ds.T @ q, p.T @ d_o


def packed_given(q, k, v, cu, scale, d_o, o_in, lse_in):
    T, hq, d = q.shape
    hkv = k.shape[1]
    G = hq // hkv
    dq = np.zeros((T, hq, d)); dk = np.zeros((T, hkv, d)); dv = np.zeros((T, hkv, d))
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        for h in range(hq):
            if a == b:
                continue
            g = h // G
            r = one_head_given(q[a:b, h], k[a:b, g], v[a:b, g], scale, d_o[a:b, h], o_in[a:b, h], lse_in[h, a:b])
            dq[a:b, h] = r[0]; dk[a:b, g] += r[1]; dv[a:b, g] += r[2]
    return dq, dk, dv
