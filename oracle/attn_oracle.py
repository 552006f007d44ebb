"""ctypes front end of the fp64 C oracle (oracle/attn_oracle.c).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg
may import this module; the product package never does, and this module imports nothing from the
product package.  The arithmetic lives in the C file; this file only compiles it, converts numpy
arrays and forwards the calls.  The definition it follows is the block-diagonal causal attention
of the paper's Sec. 2.1 (packing paragraph) and Sec. 6.1 (a packed buffer costs the sum of its
sequences), with its gradients.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (generic x86-64 code so the library runs on any host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("hyd_oracle_fwd", "hyd_oracle_bwd", "hyd_oracle_bwd_given", "hyd_oracle_rows", "hyd_oracle_cols",
                     "hyd_oracle_probs", "hyd_oracle_threads"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _f32(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x, x.ctypes.data_as(ctypes.c_void_p)


def _i32(x):
    x = np.ascontiguousarray(x, dtype=np.int32)
    return x, x.ctypes.data_as(ctypes.c_void_p)


def _out(shape):
    x = np.empty(shape, dtype=np.float64)
    return x, x.ctypes.data_as(ctypes.c_void_p)


def _dims(q, k):
    T, hq, d = q.shape
    assert k.shape[0] == T and k.shape[2] == d
    return T, hq, k.shape[1], d


def threads():
    return _load().hyd_oracle_threads()


def fwd(q, k, v, cu_seqlens, scale):
    """q[T,Hq,d], k,v[T,Hkv,d] float32 (exact input values) -> O[T,Hq,d], LSE[Hq,T], float64."""
    T, hq, hkv, d = _dims(q, k)
    q, pq = _f32(q); k, pk = _f32(k); v, pv = _f32(v); cu, pcu = _i32(cu_seqlens)
    o, po = _out((T, hq, d)); lse, pl = _out((hq, T))
    rc = _load().hyd_oracle_fwd(pq, pk, pv, pcu, len(cu) - 1, T, hq, hkv, d,
                                ctypes.c_double(scale), po, pl)
    if rc:
        raise ValueError(f"hyd_oracle_fwd failed: {rc}")
    return o, lse


def bwd(q, k, v, d_o, cu_seqlens, scale):
    """-> dQ[T,Hq,d], dK[T,Hkv,d], dV[T,Hkv,d], float64."""
    T, hq, hkv, d = _dims(q, k)
    q, pq = _f32(q); k, pk = _f32(k); v, pv = _f32(v); d_o, pdo = _f32(d_o)
    cu, pcu = _i32(cu_seqlens)
    dq, pdq = _out((T, hq, d)); dk, pdk = _out((T, hkv, d)); dv, pdv = _out((T, hkv, d))
    rc = _load().hyd_oracle_bwd(pq, pk, pv, pdo, pcu, len(cu) - 1, T, hq, hkv, d,
                                ctypes.c_double(scale), pdq, pdk, pdv)
    if rc:
        raise ValueError(f"hyd_oracle_bwd failed: {rc}")
    return dq, dk, dv


def bwd_given(q, k, v, d_o, o_in, lse_in, cu_seqlens, scale):
    """The backward as a function of what a backward call receives: the stored forward results
    o_in[T,Hq,d] (e.g. rounded to bf16) and lse_in[Hq,T] are used as given (P = exp(s - lse_in),
    D = <dO, o_in>) -> dQ, dK, dV, float64."""
    T, hq, hkv, d = _dims(q, k)
    q, pq = _f32(q); k, pk = _f32(k); v, pv = _f32(v); d_o, pdo = _f32(d_o)
    o_in, po = _f32(o_in); lse_in, pl = _f32(lse_in)
    assert o_in.shape == (T, hq, d) and lse_in.shape == (hq, T)
    cu, pcu = _i32(cu_seqlens)
    dq, pdq = _out((T, hq, d)); dk, pdk = _out((T, hkv, d)); dv, pdv = _out((T, hkv, d))
    rc = _load().hyd_oracle_bwd_given(pq, pk, pv, pdo, po, pl, pcu, len(cu) - 1, T, hq, hkv, d,
                                      ctypes.c_double(scale), pdq, pdk, pdv)
    if rc:
        raise ValueError(f"hyd_oracle_bwd_given failed: {rc}")
    return dq, dk, dv


def rows(q, k, v, d_o, cu_seqlens, scale, tok, head):
    """Sampled outputs: for packed rows tok[n] and query heads head[n] -> O rows, LSE values and
    (if d_o is not None) dQ rows."""
    T, hq, hkv, d = _dims(q, k)
    q, pq = _f32(q); k, pk = _f32(k); v, pv = _f32(v); cu, pcu = _i32(cu_seqlens)
    pdo = None
    if d_o is not None:
        d_o, pdo = _f32(d_o)
    tok, ptok = _i32(tok); head, phead = _i32(head)
    n = len(tok)
    o, po = _out((n, d)); lse, pl = _out((n,)); dq, pdq = _out((n, d))
    rc = _load().hyd_oracle_rows(pq, pk, pv, pdo, pcu, len(cu) - 1, T, hq, hkv, d,
                                 ctypes.c_double(scale), ptok, phead, n, po, pl, pdq)
    if rc:
        raise ValueError(f"hyd_oracle_rows failed: {rc}")
    return o, lse, (dq if d_o is not None else None)


def cols(q, k, v, d_o, cu_seqlens, scale, seq, kv_head, key_cols):
    """dK, dV rows of the local key indices key_cols of sequence seq and KV head kv_head."""
    T, hq, hkv, d = _dims(q, k)
    q, pq = _f32(q); k, pk = _f32(k); v, pv = _f32(v); d_o, pdo = _f32(d_o)
    cu, pcu = _i32(cu_seqlens); key_cols, pc = _i32(key_cols)
    n = len(key_cols)
    dk, pdk = _out((n, d)); dv, pdv = _out((n, d))
    rc = _load().hyd_oracle_cols(pq, pk, pv, pdo, pcu, len(cu) - 1, T, hq, hkv, d,
                                 ctypes.c_double(scale), int(seq), int(kv_head), pc, n, pdk, pdv)
    if rc:
        raise ValueError(f"hyd_oracle_cols failed: {rc}")
    return dk, dv


def probs(q, k, cu_seqlens, scale, tok, head):
    """Softmax probabilities P[i, 0..i] of one packed row."""
    T, hq, hkv, d = _dims(q, k)
    q, pq = _f32(q); k, pk = _f32(k); cu, pcu = _i32(cu_seqlens)
    s = int(np.searchsorted(cu, tok, side="right") - 1)
    p, pp = _out((int(tok) - int(cu[s]) + 1,))
    rc = _load().hyd_oracle_probs(pq, pk, pcu, len(cu) - 1, T, hq, hkv, d,
                                  ctypes.c_double(scale), int(tok), int(head), pp)
    if rc:
        raise ValueError(f"hyd_oracle_probs failed: {rc}")
    return p
