"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
sizes its workspace sanely and rejects bad arguments before touching the GPU (none of these
calls launches anything, so they run on a host without a GPU)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2412_07894_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "hyd_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hyd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2412_07894_amd import binding
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_workspace_bytes(lib):
    from paper_2412_07894_amd import binding as b
    f = b.workspace_bytes(16384, 8, 32, 32, 128, b.HYD_BF16, False)
    w = b.workspace_bytes(16384, 8, 32, 32, 128, b.HYD_BF16, True)
    assert f > 0 and f % 256 == 0 and w >= f + 4 * 16384 * 32          # backward adds D[Hq][T]
    assert b.workspace_bytes(16384, 8, 32, 5, 128, b.HYD_BF16, False) == 0   # 32 % 5
    assert b.workspace_bytes(16384, 8, 32, 32, 96, b.HYD_BF16, False) == 0   # head_dim
    assert b.workspace_bytes(-1, 8, 32, 32, 128, b.HYD_BF16, False) == 0
    assert b.workspace_bytes(0, 0, 2, 2, 64, b.HYD_FP32, True) > 0


def call_fwd(lib, **kw):
    a = dict(q=1 << 20, k=1 << 20, v=1 << 20, cu=1 << 20, nseq=2, cu_host=None, T=256, max_len=200, hq=4, hkv=2,
             d=128, scale=0.1, dt=0, o=1 << 20, lse=1 << 20, ws=1 << 20, ws_bytes=1 << 30, stream=None)
    a.update(kw)
    return lib.hyd_varlen_attn_fwd(a["q"], a["k"], a["v"], a["cu"], a["nseq"], a["cu_host"], a["T"], a["max_len"],
                                   a["hq"], a["hkv"], a["d"], a["scale"], a["dt"], a["o"], a["lse"], a["ws"],
                                   a["ws_bytes"], a["stream"])


def host_cu(vals):
    arr = (ctypes.c_int32 * len(vals))(*vals)
    return arr, ctypes.cast(arr, ctypes.c_void_p)


def test_forward_argument_errors(lib):
    """Fake non-NULL device pointers are never dereferenced: every case fails validation first."""
    OK, NULL, SHAPE, DTYPE, HEADS, HEADDIM, SEQLENS, WORKSPACE = range(8)
    assert call_fwd(lib, dt=7) == DTYPE
    assert call_fwd(lib, T=-1) == SHAPE
    assert call_fwd(lib, nseq=-2) == SHAPE
    assert call_fwd(lib, nseq=0) == SHAPE                       # tokens that belong to no sequence
    assert call_fwd(lib, hq=0) == HEADS
    assert call_fwd(lib, hq=4, hkv=3) == HEADS
    assert call_fwd(lib, d=96) == HEADDIM
    assert call_fwd(lib, d=64, q=None) == NULL                  # head_dim 64 is valid for bf16 too
    assert call_fwd(lib, d=64, T=1 << 19, max_len=1 << 19, hq=32, hkv=32) == SHAPE   # 2^19 * 32 * 64 * 2 = 2^31 bytes: the d = 64 limit
    assert call_fwd(lib, cu=None) == NULL
    assert call_fwd(lib, max_len=0) == SHAPE
    assert call_fwd(lib, max_len=257) == SHAPE
    assert call_fwd(lib, T=1 << 20, max_len=1 << 20, hq=32, hkv=32) == SHAPE     # 2^20 * 32 * 128 * 2 = 2^33 bytes
    keep, p = host_cu([0, 100, 250]);  assert call_fwd(lib, cu_host=p) == SEQLENS     # does not end at T
    keep, p = host_cu([1, 100, 256]);  assert call_fwd(lib, cu_host=p) == SEQLENS     # does not start at 0
    keep, p = host_cu([0, 260, 256]);  assert call_fwd(lib, cu_host=p) == SEQLENS     # decreasing
    keep, p = host_cu([0, 50, 256]);   assert call_fwd(lib, cu_host=p) == SHAPE       # longest 206 > max_len 200
    assert call_fwd(lib, ws=None) == WORKSPACE
    assert call_fwd(lib, ws=(1 << 20) + 8) == WORKSPACE         # misaligned
    assert call_fwd(lib, ws_bytes=16) == WORKSPACE
    assert call_fwd(lib, q=None) == NULL
    assert call_fwd(lib, lse=None) == NULL
    # empty problems are no-ops that need no pointers at all
    assert call_fwd(lib, T=0, nseq=0, q=None, k=None, v=None, cu=None, o=None, lse=None, ws=None, ws_bytes=0, max_len=0) == OK
    assert call_fwd(lib, T=0, nseq=3, q=None, k=None, v=None, cu=None, o=None, lse=None, ws=None, ws_bytes=0, max_len=0) == OK


def test_backward_argument_errors(lib):
    def bwd(**kw):
        a = dict(q=1 << 20, k=1 << 20, v=1 << 20, o=1 << 20, lse=1 << 20, do=1 << 20, cu=1 << 20, nseq=2, cu_host=None,
                 T=256, max_len=200, hq=4, hkv=2, d=128, scale=0.1, dt=0, dq=1 << 20, dk=1 << 20, dv=1 << 20,
                 ws=1 << 20, ws_bytes=1 << 30, stream=None)
        a.update(kw)
        return lib.hyd_varlen_attn_bwd(a["q"], a["k"], a["v"], a["o"], a["lse"], a["do"], a["cu"], a["nseq"], a["cu_host"],
                                       a["T"], a["max_len"], a["hq"], a["hkv"], a["d"], a["scale"], a["dt"], a["dq"],
                                       a["dk"], a["dv"], a["ws"], a["ws_bytes"], a["stream"])
    from paper_2412_07894_amd import binding as b
    assert bwd(do=None) == 1 and bwd(dv=None) == 1 and bwd(lse=None) == 1
    assert bwd(hkv=3) == 4 and bwd(d=100, dt=1) == 5 and bwd(dt=-1) == 3
    fwd_bytes = b.workspace_bytes(256, 2, 4, 2, 128, 0, False)
    assert bwd(ws_bytes=fwd_bytes) == 7                          # the backward needs the larger workspace
    assert bwd(T=0, nseq=0, max_len=0, ws=None, ws_bytes=0) == 0


def test_range_argument_errors(lib):
    """Range variants: ranges are checked against the host copies before anything is launched."""
    RANGE = 11

    def fwd_range(ranges, ranges_dev=1 << 20, cu=(0, 600, 1000), **kw):
        a = dict(q=1 << 20, k=1 << 20, v=1 << 20, cu=1 << 20, nseq=2, T=1000, max_len=600, hq=4, hkv=2, d=128,
                 scale=0.1, dt=0, o=1 << 20, lse=1 << 20, ws=1 << 20, ws_bytes=1 << 30, stream=None)
        a.update(kw)
        keep_c, pc = host_cu(list(cu)) if cu is not None else (None, None)
        keep_r, pr = host_cu([x for r in ranges for x in r])
        return lib.hyd_varlen_attn_fwd_range(a["q"], a["k"], a["v"], a["cu"], a["nseq"], pc, ranges_dev, pr, a["T"],
                                             a["max_len"], a["hq"], a["hkv"], a["d"], a["scale"], a["dt"], a["o"],
                                             a["lse"], a["ws"], a["ws_bytes"], a["stream"])
    good = [(0, 256, 0, 600), (256, 400, 0, 256)]                # ends: aligned, or at / past the sequence's end
    assert fwd_range(good, q=None) == 1                          # passes the range checks, stops at the NULL q
    assert fwd_range(good, ranges_dev=None) == 1
    assert fwd_range(good, dt=1, d=64) == 3                      # bf16 only
    assert fwd_range([(0, 256, 0, 600), (128, 400, 0, 256)]) == RANGE     # begin off the granule
    assert fwd_range([(0, 300, 0, 600), (256, 400, 0, 256)]) == RANGE     # end inside the sequence, off the granule
    assert fwd_range([(0, 256, 512, 256), (256, 400, 0, 256)]) == RANGE   # end < begin
    assert fwd_range([(-256, 256, 0, 600), (256, 400, 0, 256)]) == RANGE
    assert fwd_range([(0, 256, 0, 599), (256, 400, 0, 256)]) == RANGE     # 599 < 600 = L
    assert fwd_range([(0, 256, 0, 599), (256, 400, 0, 256)], cu=None) == RANGE   # judged against max_len = 600
    assert fwd_range([(0, 256, 256, 256), (512, 512, 0, 0)], q=None) == 1  # empty ranges are allowed

    def bwd_range(ranges, **kw):
        a = dict(q=1 << 20, dt=0)
        a.update(kw)
        keep_c, pc = host_cu([0, 600, 1000])
        keep_r, pr = host_cu([x for r in ranges for x in r])
        P = 1 << 20
        return lib.hyd_varlen_attn_bwd_range(a["q"], P, P, P, P, P, P, 2, pc, P, pr, 1000, 600, 4, 2, 128, 0.1, a["dt"],
                                             P, P, P, P, 1 << 30, None)
    assert bwd_range(good, q=None) == 1
    assert bwd_range([(0, 256, 64, 600), (256, 400, 0, 256)]) == RANGE
    assert bwd_range(good, dt=1) == 3


def test_merge_argument_errors(lib):
    P = 1 << 20
    assert lib.hyd_attn_merge(P, P, P, P, 100, 4, 128, 1, P, P, None) == 3      # bf16 only
    assert lib.hyd_attn_merge(P, P, P, P, -1, 4, 128, 0, P, P, None) == 2
    assert lib.hyd_attn_merge(P, P, P, P, 100, 0, 128, 0, P, P, None) == 4
    assert lib.hyd_attn_merge(P, P, P, P, 100, 4, 96, 0, P, P, None) == 5
    assert lib.hyd_attn_merge(P, P, None, P, 100, 4, 128, 0, P, P, None) == 1
    assert lib.hyd_attn_merge(None, None, None, None, 0, 4, 128, 0, None, None, None) == 0


def test_rope_argument_errors(lib):
    P = 1 << 20
    f = ctypes.c_float
    call = lambda **kw: lib.hyd_rope_packed(*[{**dict(x=P, cu=P, nseq=2, T=100, h=4, d=128, base=f(10000.0), inv=0, dt=0, out=P, st=None), **kw}[k]
                                              for k in ("x", "cu", "nseq", "T", "h", "d", "base", "inv", "dt", "out", "st")])
    assert call(dt=1) == 3 and call(d=96) == 5 and call(h=0) == 4
    assert call(T=-1) == 2 and call(nseq=0) == 2 and call(base=f(1.0)) == 2
    assert call(x=None) == 1 and call(cu=None) == 1 and call(out=None) == 1
    assert call(T=0, nseq=0, x=None, cu=None, out=None) == 0


def test_status_strings(lib):
    from paper_2412_07894_amd import binding as b
    seen = {b.status_string(c) for c in range(12)}
    assert len(seen) == 12 and all(s.startswith("HYD_") for s in seen)
    assert "unknown" in b.status_string(99)


def test_noalloc_forward_checks_sizes_and_arguments_before_any_hip_call(lib):
    """hyd_varlen_attn_fwd_noalloc on a host without a GPU: every argument error is reported, and
    sizes beyond the library's fixed array are HYD_ERR_WORKSPACE."""
    P = ctypes.c_void_p(1 << 20)
    f = ctypes.c_float(0.1)
    lib.hyd_varlen_attn_fwd_noalloc.restype = ctypes.c_int
    lib.hyd_varlen_attn_fwd_noalloc_max_workspace.restype = ctypes.c_size_t
    call = lambda **kw: lib.hyd_varlen_attn_fwd_noalloc(*[{**dict(q=P, k=P, v=P, cu=P, nseq=3, cuh=None, T=1000, ml=500, hq=8, hkv=2,
                                                                 d=128, sc=f, dt=0, o=P, lse=P, st=None), **kw}[k]
                                                         for k in ("q", "k", "v", "cu", "nseq", "cuh", "T", "ml", "hq", "hkv", "d", "sc", "dt", "o", "lse", "st")])
    assert lib.hyd_varlen_attn_fwd_noalloc_max_workspace() == 2 << 20
    assert call(T=-1) == 2 and call(hq=7) == 4 and call(dt=5) == 3 and call(d=96) == 5
    assert call(cu=None) == 1 and call(q=None) == 1 and call(o=None) == 1 and call(ml=2000) == 2
    bad = (ctypes.c_int32 * 4)(0, 10, 5, 1000)
    assert call(cuh=ctypes.cast(bad, ctypes.c_void_p)) == 6
    assert call(T=1 << 24, nseq=1 << 20, ml=4096) == 7          # schedule larger than the array
    assert call(T=0, nseq=0, q=None, k=None, v=None, cu=None, o=None, lse=None) == 0


def test_schedule_layout_and_status_argument_errors(lib):
    sz, ci = ctypes.c_size_t, ctypes.c_int
    h, it, cap, tile = sz(0), sz(0), ci(0), ci(0)
    lib.hyd_varlen_attn_schedule_layout.restype = ctypes.c_int
    lay = lambda T, n, hq, hkv, d, dt, bwd, which: lib.hyd_varlen_attn_schedule_layout(T, n, hq, hkv, d, dt, bwd, which, ctypes.byref(h),
                                                                                          ctypes.byref(it), ctypes.byref(cap), ctypes.byref(tile))
    assert lay(1000, 3, 8, 2, 128, 0, 0, 0) == 0 and tile.value == 256 and cap.value == 1000 // 256 + 3 + 1 and it.value > h.value
    assert lay(1000, 3, 8, 2, 128, 0, 1, 0) == 0 and tile.value == 128
    kv_items = it.value
    assert lay(1000, 3, 8, 2, 128, 0, 1, 1) == 0 and tile.value == 256 and it.value > kv_items
    assert lay(1000, 3, 8, 2, 128, 0, 0, 1) == 2 and lay(1000, 3, 8, 2, 128, 0, 1, 2) == 2 and lay(-1, 3, 8, 2, 128, 0, 1, 0) == 2
    assert lay(1000, 3, 7, 2, 128, 0, 1, 0) == 4 and lay(1000, 3, 8, 2, 96, 0, 1, 0) == 5 and lay(1000, 3, 8, 2, 128, 9, 1, 0) == 3
    assert lib.hyd_varlen_attn_schedule_layout(1000, 3, 8, 2, 128, 0, 1, 0, None, ctypes.byref(it), ctypes.byref(cap), ctypes.byref(tile)) == 1
    lib.hyd_varlen_attn_schedule_status.restype = ctypes.c_int
    P = ctypes.c_void_p(1 << 20)
    st = lambda ws, nbytes, T=1000, n=3, hq=8: lib.hyd_varlen_attn_schedule_status(ws, sz(nbytes), T, n, hq, 2, 128, 0, 0, None)
    assert st(None, 1 << 20) == 7 and st(P, 16) == 7 and st(P, 1 << 20, hq=7) == 4 and st(P, 1 << 20, T=-5) == 2
    assert st(None, 0, T=0, n=0) == 0


def test_rope_variants_argument_errors(lib):
    P = ctypes.c_void_p(1 << 20)
    f = ctypes.c_float
    lib.hyd_varlen_attn_fwd_rope.restype = ctypes.c_int
    lib.hyd_varlen_attn_bwd_rope.restype = ctypes.c_int
    fwd = lambda base, dt=0: lib.hyd_varlen_attn_fwd_rope(P, P, P, P, 3, None, 1000, 500, 8, 2, 128, f(0.1), f(base), dt, P, P, P,
                                                         ctypes.c_size_t(1 << 30), None)
    bwd = lambda base, dt=0: lib.hyd_varlen_attn_bwd_rope(P, P, P, P, P, P, P, 3, None, 1000, 500, 8, 2, 128, f(0.1), f(base), dt,
                                                         P, P, P, P, ctypes.c_size_t(1 << 30), None)
    assert fwd(1.0) == 2 and fwd(0.0) == 2 and bwd(-3.0) == 2       # the base must exceed 1
    assert fwd(10000.0, dt=1) == 3 and bwd(10000.0, dt=1) == 3     # bf16 only
    # (a call with valid arguments is never made here: these pointers are fake)
    Pn = None
    assert lib.hyd_varlen_attn_fwd_rope(Pn, P, P, P, 3, None, 1000, 500, 8, 2, 128, f(0.1), f(10000.0), 0, P, P, P,
                                        ctypes.c_size_t(1 << 30), None) == 1
