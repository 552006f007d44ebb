"""Thin Python front end of the planning calls of the C-ABI library (include/hyd_plan.h):
argument marshalling only; the fit, the packing search and the dispatcher run in the library."""
import ctypes

import numpy as np

from . import binding

EXPORTS = (
    "hyd_plan_fit_latency", "hyd_plan_latency", "hyd_plan_pack_fixed_v", "hyd_plan_v_range",
    "hyd_plan_pack", "hyd_plan_pack_ffd", "hyd_plan_dispatch",
)


class LatencyModel(ctypes.Structure):
    _fields_ = [("a", ctypes.c_double), ("b", ctypes.c_double), ("c", ctypes.c_double)]

    def as_tuple(self):
        return (self.a, self.b, self.c)


_ready = False


def _lib():
    global _ready
    lib = binding.load()
    if not _ready:
        i, i64, d = ctypes.c_int, ctypes.c_int64, ctypes.c_double
        ip, dp, i32p = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        mp = ctypes.POINTER(LatencyModel)
        lib.hyd_plan_fit_latency.restype = i
        lib.hyd_plan_fit_latency.argtypes = [dp, dp, dp, i, mp]
        lib.hyd_plan_latency.restype = d
        lib.hyd_plan_latency.argtypes = [mp, d]
        lib.hyd_plan_pack_fixed_v.restype = i
        lib.hyd_plan_pack_fixed_v.argtypes = [i32p, i, mp, i64, i, i, i64, i32p, dp, dp, ip]
        lib.hyd_plan_v_range.restype = i
        lib.hyd_plan_v_range.argtypes = [i32p, i, i64, i64, ip, ip]
        lib.hyd_plan_pack.restype = i
        lib.hyd_plan_pack.argtypes = [i32p, i, mp, i64, i64, i, i64, i32p, ip, dp, ip]
        lib.hyd_plan_pack_ffd.restype = i
        lib.hyd_plan_pack_ffd.argtypes = [i32p, i, i64, i32p, ip]
        lib.hyd_plan_dispatch.restype = i
        lib.hyd_plan_dispatch.argtypes = [i32p, i, i32p, mp, i32p, i, i32p, i, i32p, dp]
        _ready = True
    return lib


def _i32(x):
    a = np.ascontiguousarray(x, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(x):
    a = np.ascontiguousarray(x, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _model(m):
    return m if isinstance(m, LatencyModel) else LatencyModel(*m)


def _check(code):
    if code != 0:
        raise binding.HydError(code, binding.status_string(code))


def fit_latency(lengths, times, weights=None):
    l, lp = _f64(lengths)
    t, tp = _f64(times)
    if l.size != t.size:
        raise ValueError("lengths and times differ in size")
    wp = None
    if weights is not None:
        w, wp = _f64(weights)
        if w.size != l.size:
            raise ValueError("lengths and weights differ in size")
    m = LatencyModel()
    _check(_lib().hyd_plan_fit_latency(lp, tp, wp, int(l.size), ctypes.byref(m)))
    return m


def latency(model, l):
    return _lib().hyd_plan_latency(ctypes.byref(_model(model)), float(l))


def pack_fixed_v(lengths, model, max_len, n_batches, pp, node_limit=0):
    """-> (objective, assignment list, lower bound, proven_optimal)"""
    l, lp = _i32(lengths)
    out = np.zeros(max(l.size, 1), dtype=np.int32)
    obj, bnd, proven = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
    _check(_lib().hyd_plan_pack_fixed_v(lp, int(l.size), ctypes.byref(_model(model)), int(max_len), int(n_batches),
                                        int(pp), int(node_limit), out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                        ctypes.byref(obj), ctypes.byref(bnd), ctypes.byref(proven)))
    return obj.value, out[:l.size].tolist(), bnd.value, bool(proven.value)


def v_range(lengths, max_len, util_len):
    l, lp = _i32(lengths)
    lo, hi = ctypes.c_int(), ctypes.c_int()
    _check(_lib().hyd_plan_v_range(lp, int(l.size), int(max_len), int(util_len), ctypes.byref(lo), ctypes.byref(hi)))
    return lo.value, hi.value


def pack(lengths, model, max_len, util_len, pp, node_limit=0):
    """-> (objective, V, assignment list, proven_optimal)"""
    l, lp = _i32(lengths)
    out = np.zeros(max(l.size, 1), dtype=np.int32)
    v, obj, proven = ctypes.c_int(), ctypes.c_double(), ctypes.c_int()
    _check(_lib().hyd_plan_pack(lp, int(l.size), ctypes.byref(_model(model)), int(max_len), int(util_len), int(pp),
                                int(node_limit), out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                ctypes.byref(v), ctypes.byref(obj), ctypes.byref(proven)))
    return obj.value, v.value, out[:l.size].tolist(), bool(proven.value)


def pack_ffd(lengths, max_len):
    """-> (V, assignment list)"""
    l, lp = _i32(lengths)
    out = np.zeros(max(l.size, 1), dtype=np.int32)
    v = ctypes.c_int()
    _check(_lib().hyd_plan_pack_ffd(lp, int(l.size), int(max_len), out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                    ctypes.byref(v)))
    return v.value, out[:l.size].tolist()


def dispatch(lengths, J, models, pps, perms):
    """-> (cost, pipeline of every sequence); perms: [trials][B] permutations"""
    l, lp = _i32(lengths)
    j, jp = _i32(J)
    pp, ppp = _i32(pps)
    pm, pmp = _i32(np.asarray(perms, dtype=np.int32).reshape(len(perms), -1))
    ms = (LatencyModel * len(models))(*[_model(m) for m in models])
    out = np.zeros(max(l.size, 1), dtype=np.int32)
    cost = ctypes.c_double()
    _check(_lib().hyd_plan_dispatch(lp, int(l.size), jp, ms, ppp, len(models), pmp, len(perms),
                                    out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), ctypes.byref(cost)))
    return cost.value, out[:l.size].tolist()
