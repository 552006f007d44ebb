"""The library enqueues nothing but kernels on the caller's stream, so a forward+backward step can
be captured into a HIP graph and replayed: every replay must reproduce the eager results bit for
bit (no atomics, one producer per output element), with eager work between the replays."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_step_in_a_hip_graph_replays_bit_exact():
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    lengths, hq, hkv, d = [700, 1, 333, 2048, 64, 1500], 8, 2, 128
    cu_np, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", seed=11)
    T, ml = int(cu_np[-1]), max(lengths)
    dev = lambda x: torch.from_numpy(x).cuda().to(torch.bfloat16)
    qd, kd, vd, dod = dev(q), dev(k), dev(v), dev(do)
    cu = torch.from_numpy(cu_np).cuda()
    scale = 1.0 / np.sqrt(d)
    ws_f = torch.empty(binding.workspace_bytes(T, len(lengths), hq, hkv, d, binding.HYD_BF16, 0), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(binding.workspace_bytes(T, len(lengths), hq, hkv, d, binding.HYD_BF16, 1), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(qd)
    lse = torch.empty((hq, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(qd), torch.empty_like(kd), torch.empty_like(vd)

    def step():
        binding.varlen_attn_fwd(qd, kd, vd, cu, ml, scale, workspace=ws_f, out=o, lse=lse)
        binding.varlen_attn_bwd(qd, kd, vd, o, lse, dod, cu, ml, scale, workspace=ws_b, dq=dq, dk=dk, dv=dv)

    step()                                   # eager reference (also sets up per-device state)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (o, lse, dq, dk, dv)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        for t in (o, lse, dq, dk, dv):       # eager work between replays: poison the outputs
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("o", "lse", "dq", "dk", "dv"), (o, lse, dq, dk, dv), ref):
            assert torch.equal(got.view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32),
                               want.view(torch.int16 if want.dtype == torch.bfloat16 else torch.int32)), (rep, name)
