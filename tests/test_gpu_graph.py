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


def test_two_streams_with_their_own_workspaces_do_not_interfere():
    """Calls are re-entrant given distinct workspaces and outputs: two forward+backward steps of
    different batches enqueued on two streams at once give the bits of running them one by one."""
    import threading
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    import gpu_util as gu
    scale = 1.0 / np.sqrt(128)
    batches = []
    for seed, lengths in ((81, [900, 300, 2000]), (82, [64, 1500, 700, 33])):
        cu, q, k, v, do = wl.custom(lengths, 8, 4, 128, "bf16", seed)
        dev = [gu.to_dev(x, "bf16") for x in (q, k, v, do)]
        batches.append((torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda(), dev, max(lengths)))

    def run(b, stream, out):
        cu_d, (qd, kd, vd, dod), ml = b
        with torch.cuda.stream(stream):
            o, lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, ml, scale, stream=stream)
            out.extend([o, lse, *binding.varlen_attn_bwd(qd, kd, vd, o, lse, dod, cu_d, ml, scale, stream=stream)])

    ref = [[], []]
    for i, b in enumerate(batches):
        run(b, torch.cuda.current_stream(), ref[i])
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):
        got = [[], []]
        threads = [threading.Thread(target=run, args=(batches[i], streams[i], got[i])) for i in range(2)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        torch.cuda.synchronize()
        for i in range(2):
            for a, b in zip(got[i], ref[i]):
                assert torch.equal(a, b)
