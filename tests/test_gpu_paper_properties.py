"""The statements the paper makes about this path, checked on the GPU with our kernels:
  * packing 32 sequences of 1K costs far less attention time than one 32K sequence ("nearly 20x"
    on the paper's A800, Sec. 3.2; by causal pair count it is 31.97x);
  * the latency of a packed buffer is about the sum of the latencies of its sequences (Sec. 6.1);
  * forward+backward latency as a function of length is a l^2 + b l + c (App. C.2)."""
import numpy as np
import pytest
import torch

from paper_2412_07894_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

HQ, HKV, D = 32, 32, 128            # LLaMA2-7B attention shape, as in the paper's Fig. 2


def time_fwd_bwd(lengths, iters=5, warm=2):
    cu_np = wl.cu_seqlens(lengths)
    T, ml = int(cu_np[-1]), int(max(lengths))
    g = torch.Generator(device="cuda"); g.manual_seed(1)
    mk = lambda h: torch.randn((T, h, D), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    q, k, v, do = mk(HQ), mk(HKV), mk(HKV), mk(HQ)
    cu = torch.from_numpy(cu_np).cuda()
    scale = 1.0 / np.sqrt(D)
    wsf = torch.empty(binding.workspace_bytes(T, len(lengths), HQ, HKV, D, 0, 0), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(binding.workspace_bytes(T, len(lengths), HQ, HKV, D, 0, 1), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q); lse = torch.empty((HQ, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ts = []
    for it in range(warm + iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        binding.varlen_attn_fwd(q, k, v, cu, ml, scale, workspace=wsf, out=o, lse=lse)
        binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, scale, workspace=wsb, dq=dq, dk=dk, dv=dv)
        e1.record()
        torch.cuda.synchronize()
        if it >= warm:
            ts.append(e0.elapsed_time(e1))
    return float(np.median(ts))


def test_packing_32x1k_against_one_32k():
    t_packed = time_fwd_bwd([1024] * 32)
    t_single = time_fwd_bwd([32768])
    ratio = t_single / t_packed
    print(f"\n32 x 1K packed: {t_packed:.3f} ms; 1 x 32K: {t_single:.3f} ms; ratio {ratio:.1f}x "
          f"(paper: nearly 20x on A800; causal pair count: 31.97x)", flush=True)
    assert 8.0 < ratio < 40.0


def test_packed_latency_is_the_sum_of_its_sequences():
    a, b = 8192, 12288
    ta, tb, tab = time_fwd_bwd([a]), time_fwd_bwd([b]), time_fwd_bwd([a, b])
    print(f"\nt({a}) = {ta:.3f} ms, t({b}) = {tb:.3f} ms, t(packed) = {tab:.3f} ms, sum = {ta + tb:.3f} ms", flush=True)
    assert abs(tab - (ta + tb)) <= 0.15 * (ta + tb)


def test_latency_is_quadratic_in_length():
    ls = np.array([1024, 2048, 4096, 8192, 16384, 32768], dtype=np.float64)
    ts = np.array([time_fwd_bwd([int(l)]) for l in ls])
    A = np.stack([ls * ls, ls, np.ones_like(ls)], axis=1)
    coef, *_ = np.linalg.lstsq(A / ts[:, None], np.ones_like(ts), rcond=None)      # relative least squares
    fit = A @ coef
    rel = np.abs(fit - ts) / ts
    print(f"\nT(l) = a l^2 + b l + c with a = {coef[0]:.3e} ms/token^2, b = {coef[1]:.3e} ms/token, c = {coef[2]:.3e} ms; "
          f"measured {np.round(ts, 3).tolist()} ms, max relative residual {rel.max():.3f}", flush=True)
    assert rel.max() < 0.10
    assert coef[0] > 0
