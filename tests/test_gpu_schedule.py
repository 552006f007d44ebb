"""The persistent-workgroup scheduler on the GPU: the item list it builds, and how evenly the
imbalance workload (config 4: one 32768-token sequence next to 409 short ones) spreads over the
compute units.  Busy time of a CU = sum over the persistent workgroups that ran on it of
(end clock - start clock); spread = (max - min) / max over the CUs that ran a workgroup."""
import numpy as np
import pytest
import torch

from paper_2412_07894_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

KERNELS = {0: "fwd", 1: "dkdv", 2: "dq"}


def traced_run(cid, iters=3):
    cfg = wl.CONFIGS[cid]
    lengths = wl.seqlens(cid)
    cu = torch.from_numpy(wl.cu_seqlens(lengths)).cuda()
    T, ml = cfg.total_tokens, int(max(lengths))
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    mk = lambda h: torch.randn((T, h, cfg.d), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    q, k, v, do = mk(cfg.hq), mk(cfg.hkv), mk(cfg.hkv), mk(cfg.hq)
    per_kernel = 2048
    rec = torch.zeros((3 * per_kernel, 4), dtype=torch.int64, device="cuda")
    out = None
    for it in range(iters):                       # the last iteration is the one that is read
        rec.zero_()
        binding.set_wg_trace(rec)
        try:
            o, lse = binding.varlen_attn_fwd(q, k, v, cu, ml, cfg.scale)
            binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, cfg.scale)
            torch.cuda.synchronize()
        finally:
            binding.set_wg_trace(None)
        out = rec.cpu().numpy()
    return out, per_kernel, lengths, cfg


def spread_of(records):
    """records: rows {kernel<<32 | cu key, start, end, items} of one kernel (used rows only)."""
    cu_key = records[:, 0] & 0xFFFFFFFF
    busy = {}
    for key, t0, t1 in zip(cu_key, records[:, 1], records[:, 2]):
        busy[int(key)] = busy.get(int(key), 0) + int(t1 - t0)
    b = np.array(list(busy.values()), dtype=np.float64)
    return (b.max() - b.min()) / b.max(), len(busy), b


def test_config4_per_cu_busy_time_spread():
    rec, per_kernel, lengths, cfg = traced_run(4)
    for kid, name in KERNELS.items():
        r = rec[kid * per_kernel:(kid + 1) * per_kernel]
        r = r[r[:, 2] != 0]
        assert len(r) > 0, name
        spread, n_cu, busy = spread_of(r)
        span = (r[:, 2].max() - r[:, 1].min()) / 100.0          # 100 MHz clock -> microseconds
        tail = (r[:, 2].max() - r[:, 2].min()) / 100.0
        print(f"\nconfig 4 {name}: {len(r)} workgroups on {n_cu} CUs, kernel span {span:.0f} us, "
              f"per-CU busy spread {100 * spread:.2f} %, idle tail (last end - first end) {tail:.0f} us, "
              f"items per workgroup min/max {r[:, 3].min()}/{r[:, 3].max()}", flush=True)
        assert n_cu == 256
        assert spread <= 0.10, f"{name}: per-CU busy-time spread {spread:.3f}"


def test_item_count_is_the_triangular_tile_count():
    """Cost is sum S_i^2, not (sum S_i)^2: the work list holds sum_s ceil(L_s / tile) items, and
    the per-workgroup item counters add up to items x heads."""
    rec, per_kernel, lengths, cfg = traced_run(2, iters=1)
    for kid, tile, heads in ((0, 256, cfg.hq), (1, 128, cfg.hkv), (2, 256, cfg.hq)):
        r = rec[kid * per_kernel:(kid + 1) * per_kernel]
        done = int(r[:, 3].sum())
        want = sum(-(-L // tile) for L in lengths) * heads
        assert done == want, (KERNELS[kid], done, want)
