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


def test_level_arrays_in_global_memory_when_max_seqlen_is_a_loose_bound():
    """A caller may pass max_seqlen = T.  With more than half a million tokens that is more
    levels than the schedule prelude keeps in LDS, so it works in the workspace instead: same
    item list, same results (sampled oracle rows and keys)."""
    from oracle import attn_oracle as orc
    import gpu_util as gu
    rng = np.random.default_rng(11)
    lengths = [int(x) for x in rng.integers(200, 1500, size=1300)]
    lengths[17] = 5000
    hq, hkv, d = 2, 1, 128
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 61)
    T = int(cu[-1])
    assert T > 4096 * 256, "the case must exceed the level count the prelude holds in LDS, for both tile sizes"
    print(f"\nloose max_seqlen: T={T} sequences={len(lengths)}", flush=True)
    scale = 1.0 / np.sqrt(d)
    qd, kd, vd, dod = (gu.to_dev(x, "bf16") for x in (q, k, v, do))
    cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    o, lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, T, scale)                 # no host copy either
    dq, dk, dv = binding.varlen_attn_bwd(qd, kd, vd, o, lse, dod, cu_d, T, scale)
    o2, lse2 = binding.varlen_attn_fwd(qd, kd, vd, cu_d, max(lengths), scale, cu_seqlens_host=[int(x) for x in cu])
    dq2, dk2, dv2 = binding.varlen_attn_bwd(qd, kd, vd, o2, lse2, dod, cu_d, max(lengths), scale)
    torch.cuda.synchronize()
    for a, b in ((o, o2), (lse, lse2), (dq, dq2), (dk, dk2), (dv, dv2)):
        assert torch.equal(a, b)               # the bound changes the schedule, never a bit of the result
    toks, heads = gu.sample_rows(cu, hq, rng, 80)
    ro, rlse, rdq = orc.rows(q, k, v, do, cu, scale, toks, heads)
    ti, hi = torch.from_numpy(toks.astype(np.int64)).cuda(), torch.from_numpy(heads.astype(np.int64)).cuda()
    gu.check("o[rows]", gu.to_np(o[ti, hi]), ro, "bf16")
    gu.check("lse[rows]", gu.to_np(lse[hi, ti]), rlse, "bf16")
    gu.check("dq[rows]", gu.to_np(dq[ti, hi]), rdq, "bf16")
    s = 17
    cols = np.array([0, 1, 127, 128, 2500, 4998, 4999], dtype=np.int32)
    rk, rv = orc.cols(q, k, v, do, cu, scale, s, 0, cols)
    idx = torch.from_numpy((cu[s] + cols).astype(np.int64)).cuda()
    gu.check("dk[keys]", gu.to_np(dk[idx, 0]), rk, "bf16")
    gu.check("dv[keys]", gu.to_np(dv[idx, 0]), rv, "bf16")


def _item_lists_match(lengths, hq, hkv, d=128):
    """Runs forward and backward, reads the three item lists back from the workspaces and compares
    them with the reference enumeration: the same records level by level (the order inside a
    level is free), levels never increasing along the list.  Integer work: exact."""
    from oracle import sched_oracle as so
    cu_np = wl.cu_seqlens(lengths)
    T, nseq, ml = int(cu_np[-1]), len(lengths), int(max(lengths))
    cu = torch.from_numpy(cu_np).cuda()
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    mk = lambda h: torch.randn((T, h, d), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    q, k, v, do = mk(hq), mk(hkv), mk(hkv), mk(hq)
    code = binding.HYD_BF16
    ws_f = torch.empty(binding.workspace_bytes(T, nseq, hq, hkv, d, code, 0), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(binding.workspace_bytes(T, nseq, hq, hkv, d, code, 1), dtype=torch.uint8, device="cuda")
    o, lse = binding.varlen_attn_fwd(q, k, v, cu, ml, 0.088, workspace=ws_f)
    binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, 0.088, workspace=ws_b)
    torch.cuda.synchronize()
    assert binding.schedule_status(ws_f, T, nseq, hq, hkv, d, code, 0) == 0
    assert binding.schedule_status(ws_b, T, nseq, hq, hkv, d, code, 1) == 0
    for ws, is_bwd, which, name in ((ws_f, 0, 0, "forward"), (ws_b, 1, 0, "dK/dV"), (ws_b, 1, 1, "dQ")):
        tile, rec = binding.schedule_items(ws, T, nseq, hq, hkv, d, code, is_bwd, which)
        ref = so.records(lengths, tile)
        print(f"{name}: tile {tile}, {len(rec)} items (reference {len(ref)}), top level {rec[0][1] if len(rec) else 0}", flush=True)
        assert len(rec) == len(ref), name
        levels = rec[:, 1]
        assert np.all(levels[:-1] >= levels[1:]), name
        assert sorted(map(tuple, rec.tolist())) == sorted(ref), name


def test_item_lists_equal_the_reference_enumeration_config1_lengths():
    _item_lists_match([1, 7, 64, 184], 2, 2)


def test_item_lists_equal_the_reference_enumeration_config4():
    _item_lists_match(wl.seqlens(4), 8, 2)            # the sequence structure of configuration 4, fewer heads


def test_item_lists_with_empty_sequences_and_tile_boundaries():
    _item_lists_match([0, 128, 129, 0, 256, 257, 1, 1000, 0], 4, 4)


def test_prelude_reports_what_it_saw_in_device_seqlens():
    """Without a host copy of cu_seqlens the call cannot validate it; the prelude leaves its
    findings in the workspace and hyd_varlen_attn_schedule_status reads them back."""
    lengths = [300, 700, 20]
    cu_np = wl.cu_seqlens(lengths)
    T, nseq, hq, hkv, d = int(cu_np[-1]), 3, 2, 1, 128
    g = torch.Generator(device="cuda"); g.manual_seed(12)
    mk = lambda h: torch.randn((T, h, d), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    q, k, v = mk(hq), mk(hkv), mk(hkv)
    code = binding.HYD_BF16
    ws = torch.empty(binding.workspace_bytes(T, nseq, hq, hkv, d, code, 0), dtype=torch.uint8, device="cuda")
    cu = torch.from_numpy(cu_np).cuda()
    binding.varlen_attn_fwd(q, k, v, cu, 700, 0.1, workspace=ws)
    assert binding.schedule_status(ws, T, nseq, hq, hkv, d, code, 0) == 0
    # max_seqlen below the longest sequence: items only up to the bound, reported as HYD_ERR_SHAPE
    binding.varlen_attn_fwd(q, k, v, cu, 256, 0.1, workspace=ws)
    assert binding.schedule_status(ws, T, nseq, hq, hkv, d, code, 0) == 2
    # a cu_seqlens that does not end at T (rows stay inside the buffers: the last entry is smaller)
    short = torch.from_numpy(np.array([0, 300, 1000, 1010], dtype=np.int32)).cuda()
    binding.varlen_attn_fwd(q, k, v, short, 700, 0.1, workspace=ws)
    assert binding.schedule_status(ws, T, nseq, hq, hkv, d, code, 0) == 6
    binding.varlen_attn_fwd(q, k, v, cu, 700, 0.1, workspace=ws)         # and a good call clears the flags again
    assert binding.schedule_status(ws, T, nseq, hq, hkv, d, code, 0) == 0
