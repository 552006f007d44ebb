"""Thin Python front end of the C-ABI library (include/hyd_attn.h): argument marshalling only.
PyTorch supplies device memory and the current HIP stream; every step of the computation runs in
the library's HIP kernels.  There is no fallback: if the library is missing or a call fails, an
exception is raised."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhyd_attn.so")
HYD_BF16, HYD_FP32 = 0, 1
_lib = None

EXPORTS = (
    "hyd_status_string", "hyd_varlen_attn_workspace_bytes", "hyd_varlen_attn_fwd",
    "hyd_varlen_attn_bwd", "hyd_enable_kernel_timing", "hyd_kernel_times", "hyd_set_wg_trace",
    "hyd_varlen_attn_fwd_range", "hyd_varlen_attn_bwd_range", "hyd_attn_merge", "hyd_rope_packed",
    "hyd_varlen_attn_fwd_noalloc", "hyd_varlen_attn_fwd_noalloc_max_workspace",
    "hyd_varlen_attn_schedule_status", "hyd_varlen_attn_schedule_layout",
    "hyd_varlen_attn_fwd_rope", "hyd_varlen_attn_bwd_rope",
)
RANGE_ALIGN = 256   # HYD_RANGE_ALIGN of the header


class HydError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"hyd_attn error {code}: {msg}")
        self.code = code


def load():
    """Load libhyd_attn.so (built by paper_2412_07894_amd/build.py; never built implicitly here)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python paper_2412_07894_amd/build.py` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ip, i, f, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.hyd_status_string.restype = ctypes.c_char_p
    lib.hyd_status_string.argtypes = [i]
    lib.hyd_varlen_attn_workspace_bytes.restype = sz
    lib.hyd_varlen_attn_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    lib.hyd_varlen_attn_fwd.restype = i
    lib.hyd_varlen_attn_fwd.argtypes = [vp, vp, vp, ip, i, ip, i, i, i, i, i, f, i, vp, vp, vp, sz, vp]
    lib.hyd_varlen_attn_fwd_noalloc.restype = i
    lib.hyd_varlen_attn_fwd_noalloc.argtypes = [vp, vp, vp, ip, i, ip, i, i, i, i, i, f, i, vp, vp, vp]
    lib.hyd_varlen_attn_fwd_noalloc_max_workspace.restype = sz
    lib.hyd_varlen_attn_fwd_noalloc_max_workspace.argtypes = []
    lib.hyd_varlen_attn_schedule_status.restype = i
    lib.hyd_varlen_attn_schedule_status.argtypes = [vp, sz, i, i, i, i, i, i, i, vp]
    lib.hyd_varlen_attn_schedule_layout.restype = i
    lib.hyd_varlen_attn_schedule_layout.argtypes = [i, i, i, i, i, i, i, i, ctypes.POINTER(sz), ctypes.POINTER(sz),
                                                    ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.hyd_varlen_attn_fwd_rope.restype = i
    lib.hyd_varlen_attn_fwd_rope.argtypes = [vp, vp, vp, ip, i, ip, i, i, i, i, i, f, f, i, vp, vp, vp, sz, vp]
    lib.hyd_varlen_attn_bwd_rope.restype = i
    lib.hyd_varlen_attn_bwd_rope.argtypes = [vp, vp, vp, vp, vp, vp, ip, i, ip, i, i, i, i, i, f, f, i,
                                             vp, vp, vp, vp, sz, vp]
    lib.hyd_varlen_attn_bwd.restype = i
    lib.hyd_varlen_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, ip, i, ip, i, i, i, i, i, f, i,
                                        vp, vp, vp, vp, sz, vp]
    lib.hyd_varlen_attn_fwd_range.restype = i
    lib.hyd_varlen_attn_fwd_range.argtypes = [vp, vp, vp, ip, i, ip, ip, ip, i, i, i, i, i, f, i, vp, vp, vp, sz, vp]
    lib.hyd_varlen_attn_bwd_range.restype = i
    lib.hyd_varlen_attn_bwd_range.argtypes = [vp, vp, vp, vp, vp, vp, ip, i, ip, ip, ip, i, i, i, i, i, f, i,
                                              vp, vp, vp, vp, sz, vp]
    lib.hyd_attn_merge.restype = i
    lib.hyd_attn_merge.argtypes = [vp, vp, vp, vp, i, i, i, i, vp, vp, vp]
    lib.hyd_rope_packed.restype = i
    lib.hyd_rope_packed.argtypes = [vp, ip, i, i, i, i, f, i, i, vp, vp]
    lib.hyd_enable_kernel_timing.restype = None
    lib.hyd_enable_kernel_timing.argtypes = [i]
    lib.hyd_kernel_times.restype = i
    lib.hyd_kernel_times.argtypes = [ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float), i]
    lib.hyd_set_wg_trace.restype = None
    lib.hyd_set_wg_trace.argtypes = [vp, i]
    _lib = lib
    return lib


def status_string(code):
    return load().hyd_status_string(int(code)).decode()


def _check(code):
    if code != 0:
        raise HydError(code, status_string(code))


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return HYD_BF16
    if t.dtype == torch.float32:
        return HYD_FP32
    raise TypeError(f"unsupported dtype {t.dtype}")


def workspace_bytes(total_tokens, num_seqs, hq, hkv, head_dim, dtype_code, is_bwd):
    return int(load().hyd_varlen_attn_workspace_bytes(total_tokens, num_seqs, hq, hkv, head_dim,
                                                      dtype_code, int(is_bwd)))


def _workspace(nbytes, device):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _host_ptr(cu_host):
    if cu_host is None:
        return None, None
    keep = (ctypes.c_int32 * len(cu_host))(*[int(x) for x in cu_host])
    return keep, ctypes.cast(keep, ctypes.c_void_p)


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def varlen_attn_fwd(q, k, v, cu_seqlens, max_seqlen, softmax_scale, cu_seqlens_host=None,
                    workspace=None, stream=None, out=None, lse=None, rope_base=None):
    """q[T,Hq,d], k,v[T,Hkv,d] contiguous device tensors (bf16 or fp32); cu_seqlens int32 device
    tensor [num_seqs+1].  Returns (o[T,Hq,d], lse[Hq,T] fp32).  With rope_base the call is
    hyd_varlen_attn_fwd_rope: q unrotated (rotated inside the kernel), k already rotated."""
    lib = load()
    T, hq, d = q.shape
    hkv = k.shape[1]
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_contiguous()
    dt = _dtype_code(q)
    nseq = cu_seqlens.numel() - 1
    o = torch.empty_like(q) if out is None else out
    lse = torch.empty((hq, T), dtype=torch.float32, device=q.device) if lse is None else lse
    need = workspace_bytes(T, nseq, hq, hkv, d, dt, False)
    ws = _workspace(need, q.device) if workspace is None else workspace
    keep, hp = _host_ptr(cu_seqlens_host)
    if rope_base is None:
        _check(lib.hyd_varlen_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), cu_seqlens.data_ptr(), nseq,
                                       hp, T, int(max_seqlen), hq, hkv, d, float(softmax_scale), dt,
                                       o.data_ptr(), lse.data_ptr(), ws.data_ptr(), ws.numel(),
                                       _stream_ptr(stream)))
    else:
        _check(lib.hyd_varlen_attn_fwd_rope(q.data_ptr(), k.data_ptr(), v.data_ptr(), cu_seqlens.data_ptr(), nseq,
                                            hp, T, int(max_seqlen), hq, hkv, d, float(softmax_scale), float(rope_base), dt,
                                            o.data_ptr(), lse.data_ptr(), ws.data_ptr(), ws.numel(),
                                            _stream_ptr(stream)))
    return o, lse


def varlen_attn_fwd_noalloc(q, k, v, cu_seqlens, max_seqlen, softmax_scale, out, lse, cu_seqlens_host=None, stream=None):
    """The forward without a workspace: the library keeps the schedule in an array of its own
    (see the header); `out` and `lse` are caller-owned, nothing is allocated here or there."""
    T, hq, d = q.shape
    hkv = k.shape[1]
    for t in (q, k, v, out, lse, cu_seqlens):
        assert t.is_contiguous()
    assert out.shape == q.shape and out.dtype == q.dtype and lse.dtype == torch.float32 and lse.shape == (hq, T)
    keep, hp = _host_ptr(cu_seqlens_host)
    _check(load().hyd_varlen_attn_fwd_noalloc(q.data_ptr(), k.data_ptr(), v.data_ptr(), cu_seqlens.data_ptr(),
                                              cu_seqlens.numel() - 1, hp, T, int(max_seqlen), hq, hkv, d,
                                              float(softmax_scale), _dtype_code(q), out.data_ptr(), lse.data_ptr(),
                                              _stream_ptr(stream)))
    return out, lse


def varlen_attn_bwd(q, k, v, o, lse, d_o, cu_seqlens, max_seqlen, softmax_scale, cu_seqlens_host=None,
                    workspace=None, stream=None, dq=None, dk=None, dv=None, rope_base=None):
    """Returns (dq, dk, dv) with the shapes and dtype of q, k, v.  With rope_base the call is
    hyd_varlen_attn_bwd_rope: q unrotated, k rotated; dq is for the unrotated q, dk for the rotated k."""
    lib = load()
    T, hq, d = q.shape
    hkv = k.shape[1]
    for t in (q, k, v, o, d_o, lse):
        assert t.is_contiguous()
    dt = _dtype_code(q)
    nseq = cu_seqlens.numel() - 1
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = workspace_bytes(T, nseq, hq, hkv, d, dt, True)
    ws = _workspace(need, q.device) if workspace is None else workspace
    keep, hp = _host_ptr(cu_seqlens_host)
    if rope_base is None:
        _check(lib.hyd_varlen_attn_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                       d_o.data_ptr(), cu_seqlens.data_ptr(), nseq, hp, T, int(max_seqlen),
                                       hq, hkv, d, float(softmax_scale), dt, dq.data_ptr(), dk.data_ptr(),
                                       dv.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    else:
        _check(lib.hyd_varlen_attn_bwd_rope(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                            d_o.data_ptr(), cu_seqlens.data_ptr(), nseq, hp, T, int(max_seqlen),
                                            hq, hkv, d, float(softmax_scale), float(rope_base), dt, dq.data_ptr(),
                                            dk.data_ptr(), dv.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return dq, dk, dv


def _ranges_args(ranges, nseq, device):
    """ranges: sequence of (q_begin, q_end, kv_begin, kv_end) per sequence -> (device tensor, host
    array kept alive, host pointer)."""
    flat = [int(x) for r in ranges for x in r]
    assert len(flat) == 4 * nseq, "one (q_begin, q_end, kv_begin, kv_end) per sequence"
    dev = torch.tensor(flat, dtype=torch.int32, device=device) if nseq else torch.zeros(4, dtype=torch.int32, device=device)
    keep = (ctypes.c_int32 * max(len(flat), 1))(*flat)
    return dev, keep, ctypes.cast(keep, ctypes.c_void_p)


def varlen_attn_fwd_range(q, k, v, cu_seqlens, ranges, max_seqlen, softmax_scale, out, lse,
                          cu_seqlens_host=None, workspace=None, stream=None):
    """One visit of a key range to a query range for every sequence (see the header).  `out` and
    `lse` are caller-owned and only the rows of the query ranges are written."""
    lib = load()
    T, hq, d = q.shape
    hkv = k.shape[1]
    for t in (q, k, v, out, lse, cu_seqlens):
        assert t.is_contiguous()
    assert lse.dtype == torch.float32 and lse.shape == (hq, T) and out.shape == q.shape and out.dtype == q.dtype
    dt = _dtype_code(q)
    nseq = cu_seqlens.numel() - 1
    need = workspace_bytes(T, nseq, hq, hkv, d, dt, False)
    ws = _workspace(need, q.device) if workspace is None else workspace
    keep, hp = _host_ptr(cu_seqlens_host)
    rdev, rkeep, rhp = _ranges_args(ranges, nseq, q.device)
    _check(lib.hyd_varlen_attn_fwd_range(q.data_ptr(), k.data_ptr(), v.data_ptr(), cu_seqlens.data_ptr(), nseq,
                                         hp, rdev.data_ptr(), rhp, T, int(max_seqlen), hq, hkv, d,
                                         float(softmax_scale), dt, out.data_ptr(), lse.data_ptr(),
                                         ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return out, lse


def varlen_attn_bwd_range(q, k, v, o, lse, d_o, cu_seqlens, ranges, max_seqlen, softmax_scale, dq, dk, dv,
                          cu_seqlens_host=None, workspace=None, stream=None):
    """Partial gradients of one visit; o and lse are the merged forward results.  dq / dk / dv are
    caller-owned; only the rows of the query (dq) and key (dk, dv) ranges are written."""
    lib = load()
    T, hq, d = q.shape
    hkv = k.shape[1]
    for t in (q, k, v, o, d_o, lse, dq, dk, dv, cu_seqlens):
        assert t.is_contiguous()
    assert dq.shape == q.shape and dk.shape == k.shape and dv.shape == v.shape
    dt = _dtype_code(q)
    nseq = cu_seqlens.numel() - 1
    need = workspace_bytes(T, nseq, hq, hkv, d, dt, True)
    ws = _workspace(need, q.device) if workspace is None else workspace
    keep, hp = _host_ptr(cu_seqlens_host)
    rdev, rkeep, rhp = _ranges_args(ranges, nseq, q.device)
    _check(lib.hyd_varlen_attn_bwd_range(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                         d_o.data_ptr(), cu_seqlens.data_ptr(), nseq, hp, rdev.data_ptr(), rhp,
                                         T, int(max_seqlen), hq, hkv, d, float(softmax_scale), dt,
                                         dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ws.data_ptr(), ws.numel(),
                                         _stream_ptr(stream)))
    return dq, dk, dv


def attn_merge(o_a, lse_a, o_b, lse_b, out=None, lse_out=None, stream=None):
    """Log-sum-exp merge of two partial results; out / lse_out may be either input pair."""
    T, hq, d = o_a.shape
    out = torch.empty_like(o_a) if out is None else out
    lse_out = torch.empty_like(lse_a) if lse_out is None else lse_out
    for t in (o_a, lse_a, o_b, lse_b, out, lse_out):
        assert t.is_contiguous()
    assert o_b.shape == o_a.shape and lse_a.shape == (hq, T) and lse_b.shape == (hq, T)
    _check(load().hyd_attn_merge(o_a.data_ptr(), lse_a.data_ptr(), o_b.data_ptr(), lse_b.data_ptr(), T, hq, d,
                                 _dtype_code(o_a), out.data_ptr(), lse_out.data_ptr(), _stream_ptr(stream)))
    return out, lse_out


def rope_packed(x, cu_seqlens, base=10000.0, inverse=False, out=None, stream=None):
    """Rotary embedding with per-sequence position reset on x[T,H,d] (bf16); out may be x."""
    T, h, d = x.shape
    out = torch.empty_like(x) if out is None else out
    assert x.is_contiguous() and out.is_contiguous() and out.shape == x.shape and out.dtype == x.dtype
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_contiguous()
    _check(load().hyd_rope_packed(x.data_ptr(), cu_seqlens.data_ptr(), cu_seqlens.numel() - 1, T, h, d, float(base),
                                  int(bool(inverse)), _dtype_code(x), out.data_ptr(), _stream_ptr(stream)))
    return out


def enable_kernel_timing(on):
    load().hyd_enable_kernel_timing(int(bool(on)))


def kernel_times(cap=8192):
    """[(kernel name, milliseconds)] in launch order of every kernel enqueued since timing was
    enabled or since the previous call of this function; synchronises on them and empties the list."""
    names = (ctypes.c_char_p * cap)()
    ms = (ctypes.c_float * cap)()
    n = load().hyd_kernel_times(names, ms, cap)
    return [(names[i].decode(), float(ms[i])) for i in range(n)]


def set_wg_trace(records):
    """records: int64 device tensor [3 * per_kernel, 4] (or None to switch the trace off)."""
    if records is None:
        load().hyd_set_wg_trace(None, 0)
    else:
        assert records.dtype == torch.int64 and records.is_contiguous() and records.shape[1] == 4
        load().hyd_set_wg_trace(records.data_ptr(), records.shape[0])


def schedule_status(workspace, total_tokens, num_seqs, hq, hkv, head_dim, dtype_code, is_bwd, stream=None):
    """Status code of what the last call's schedule prelude saw in the device cu_seqlens
    (synchronises the stream): 0, HYD_ERR_SHAPE (2) or HYD_ERR_SEQLENS (6)."""
    return int(load().hyd_varlen_attn_schedule_status(workspace.data_ptr(), workspace.numel(), total_tokens, num_seqs, hq, hkv,
                                                      head_dim, dtype_code, int(is_bwd), _stream_ptr(stream)))


def schedule_items(workspace, total_tokens, num_seqs, hq, hkv, head_dim, dtype_code, is_bwd, which):
    """The item list a finished call left in `workspace`: (tile, int array [n, 4] of (sequence,
    level, first packed row, length)), copied to the host."""
    hdr, items, cap, tile = ctypes.c_size_t(0), ctypes.c_size_t(0), ctypes.c_int(0), ctypes.c_int(0)
    _check(load().hyd_varlen_attn_schedule_layout(total_tokens, num_seqs, hq, hkv, head_dim, dtype_code, int(is_bwd), int(which),
                                                  ctypes.byref(hdr), ctypes.byref(items), ctypes.byref(cap), ctypes.byref(tile)))
    torch.cuda.synchronize()
    n = int(workspace[hdr.value:hdr.value + 4].view(torch.int32).item())
    assert 0 <= n <= cap.value
    rec = workspace[items.value:items.value + 16 * n].view(torch.int32).reshape(n, 4).cpu().numpy()
    return tile.value, rec
