"""Full-size parity on the benchmark configurations 2-5, in the launch configuration bench.py
times (one call over the concatenation of all buffers).  The fp64 oracle cannot run these sizes
in full, so it computes sampled outputs one by one: rows of O, LSE and dQ (each needs only its
own sequence prefix) and rows of dK and dV for sampled keys of chosen (sequence, KV head) pairs.
Samples always include sequence starts and ends, tile boundaries and the longest sequence, whose
sampled keys reach down to key 0 (the keys with the longest sums).  Every check prints the number
of elements it covers and their share of the tensor."""
import time

import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def run_config(cid, n_rows=2000, col_cases=3, n_random_keys=48):
    cfg = wl.CONFIGS[cid]
    lengths = wl.seqlens(cid)
    cu = wl.cu_seqlens(lengths)
    T = cfg.total_tokens
    t0 = time.time()
    q = wl.normal_tensor(cid, "q", T, cfg.hq, cfg.d, cfg.dtype)
    k = wl.normal_tensor(cid, "k", T, cfg.hkv, cfg.d, cfg.dtype)
    v = wl.normal_tensor(cid, "v", T, cfg.hkv, cfg.d, cfg.dtype)
    do = wl.normal_tensor(cid, "do", T, cfg.hq, cfg.d, cfg.dtype)
    print(f"\nconfig {cid}: T={T} seqs={len(lengths)} longest={max(lengths)} inputs in {time.time() - t0:.1f}s", flush=True)
    dev = lambda x: torch.from_numpy(x).cuda().to(torch.bfloat16)
    qd, kd, vd, dod = dev(q), dev(k), dev(v), dev(do)
    cu_d = torch.from_numpy(cu).cuda()
    ml = int(max(lengths))
    o, lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, ml, cfg.scale, cu_seqlens_host=list(cu))
    dq, dk, dv = binding.varlen_attn_bwd(qd, kd, vd, o, lse, dod, cu_d, ml, cfg.scale, cu_seqlens_host=list(cu))
    torch.cuda.synchronize()
    for t in (o, lse, dq, dk, dv):
        assert bool(torch.isfinite(t).all())
    rng = np.random.default_rng(100 + cid)
    toks, heads = gu.sample_rows(cu, cfg.hq, rng, n_rows)
    t0 = time.time()
    ro, rlse, rdq = orc.rows(q, k, v, do, cu, cfg.scale, toks, heads)
    print(f"oracle: {len(toks)} sampled rows in {time.time() - t0:.1f}s", flush=True)
    ti, hi = torch.from_numpy(toks.astype(np.int64)).cuda(), torch.from_numpy(heads.astype(np.int64)).cuda()
    failures = []
    n_q, n_kv = T * cfg.hq * cfg.d, T * cfg.hkv * cfg.d
    print(f"covered: {ro.size} of {n_q} elements of O and of dQ ({ro.size / n_q:.2e}), "
          f"{rlse.size} of {T * cfg.hq} of LSE ({rlse.size / (T * cfg.hq):.2e})", flush=True)
    gu.check("o[rows]", gu.to_np(o[ti, hi]), ro, "bf16", failures=failures)
    gu.check("lse[rows]", gu.to_np(lse[hi, ti]), rlse, "bf16", failures=failures)
    gu.check("dq[rows]", gu.to_np(dq[ti, hi]), rdq, "bf16", failures=failures)
    # dK / dV of sampled keys: the longest sequence, a mid-sized one and a short one
    lens = np.diff(cu)
    order = np.argsort(-lens)
    picks = [int(order[0]), int(order[len(order) // 2]), int(order[-1])][:col_cases]
    gk, gv, rk, rv = [], [], [], []
    for n, s in enumerate(picks):
        L = int(lens[s])
        g = int(rng.integers(0, cfg.hkv))
        # key 0 is always in: the cost is that of every row of the sequence for the group's
        # heads whatever the keys are, so more keys are nearly free
        cols = {0, 1, 2, 31, 32, 63, 64, 127, 128, 255, 256, L // 3, L // 2, L - 129, L - 33, L - 2, L - 1}
        # the longest sequence gets many more: its keys have the longest sums, and every row of the
        # sequence is evaluated for the group's heads anyway
        cols |= {int(c) for c in rng.integers(0, L, 1024 if n == 0 else n_random_keys)}
        cols = np.array(sorted(cols & set(range(L))), dtype=np.int32)
        t0 = time.time()
        a, b = orc.cols(q, k, v, do, cu, cfg.scale, s, g, cols)
        print(f"oracle: dK/dV of {len(cols)} keys of sequence {s} (L={L}), KV head {g} in {time.time() - t0:.1f}s", flush=True)
        idx = torch.from_numpy((cu[s] + cols).astype(np.int64)).cuda()
        gk.append(gu.to_np(dk[idx, g])); gv.append(gu.to_np(dv[idx, g])); rk.append(a); rv.append(b)
    rk, rv = np.concatenate(rk), np.concatenate(rv)
    print(f"covered: {rk.size} of {n_kv} elements of dK and of dV ({rk.size / n_kv:.2e})", flush=True)
    gu.check("dk[keys]", np.concatenate(gk), rk, "bf16", failures=failures)
    gu.check("dv[keys]", np.concatenate(gv), rv, "bf16", failures=failures)
    assert not failures, "\n".join(failures)


@pytest.mark.parametrize("cid", [2, 3, 4, 5])
def test_config_sampled_parity(cid):
    run_config(cid)
