"""The forward entry point that allocates nothing (hyd_varlen_attn_fwd_noalloc: schedule in an
array inside the library) against hyd_varlen_attn_fwd on the same inputs: identical bits, on two
calls in a row of which the second is smaller (the array keeps the first call's contents), and
the size limit is an error."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def both(lengths, hq, hkv, d, seed):
    cu, q, k, v, _ = wl.custom(lengths, hq, hkv, d, "bf16", seed)
    scale = 1.0 / float(np.sqrt(d))
    qd, kd, vd = (gu.to_dev(x, "bf16") for x in (q, k, v))
    cu_d = torch.from_numpy(cu).cuda()
    T = int(cu[-1])
    ref_o, ref_lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, max(lengths), scale, cu_seqlens_host=list(cu))
    out = torch.full((T, hq, d), 5.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((hq, T), 5.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.varlen_attn_fwd_noalloc(qd, kd, vd, cu_d, max(lengths), scale, out, lse, cu_seqlens_host=list(cu))
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert torch.equal(out, ref_o) and torch.equal(lse, ref_lse)


def test_noalloc_forward_twice_second_call_smaller():
    print("\nno-alloc forward: 3 sequences / 6 heads, then 2 sequences / 2 heads", flush=True)
    both([700, 129, 2100, 1], 6, 3, 128, seed=91)
    both([300, 45], 2, 1, 128, seed=92)          # fewer items, sequences and heads than the array still holds
    both([64, 0, 513], 4, 4, 64, seed=93)


def test_noalloc_size_limit_is_an_error():
    lib = binding.load()
    cap = lib.hyd_varlen_attn_fwd_noalloc_max_workspace()
    assert cap == 2 << 20
    T, nseq = 1 << 24, 1 << 20
    assert binding.workspace_bytes(T, nseq, 8, 8, 128, binding.HYD_BF16, 0) > cap
    P = ctypes.c_void_p(1 << 20)
    rc = lib.hyd_varlen_attn_fwd_noalloc(P, P, P, P, nseq, None, T, 4096, 8, 8, 128, ctypes.c_float(0.1), 0, P, P, None)
    assert rc == 7 and "WORKSPACE" in binding.status_string(rc)


def test_noalloc_forward_in_a_hip_graph():
    """What the entry point is for: captured into a HIP graph (no allocation may happen under
    capture) and replayed, with eager work between the replays, it reproduces the eager bits."""
    lengths, hq, hkv, d = [700, 1, 333, 1500], 4, 2, 128
    cu, q, k, v, _ = wl.custom(lengths, hq, hkv, d, "bf16", seed=94)
    scale = 1.0 / float(np.sqrt(d))
    qd, kd, vd = (gu.to_dev(x, "bf16") for x in (q, k, v))
    cu_d = torch.from_numpy(cu).cuda()
    T = int(cu[-1])
    ref_o, ref_lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, max(lengths), scale)
    out = torch.empty((T, hq, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((hq, T), dtype=torch.float32, device="cuda")
    run = lambda: binding.varlen_attn_fwd_noalloc(qd, kd, vd, cu_d, max(lengths), scale, out, lse)
    run()                                            # sets up the per-device state outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        out.fill_(float("nan")); lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_o) and torch.equal(lse, ref_lse), rep
