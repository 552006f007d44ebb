#!/usr/bin/env python3
"""Context parallelism seen from one GPU (Hydraulis, arXiv 2412.07894: CP is the third axis of
the parallel schemes <TP, PP, CP>, Sec. 2.1; App. C.1 prices its memory).  Under a CP degree of N
every sequence of a packed buffer is cut into N chunks; rank r owns query chunk r and meets the
key/value chunks 0..r one after the other (later chunks are hidden from it by causality).  One
GPU can show exactly one rank's share at its real shape: this module times, through the range
variants of the library, every visit of one rank - forward and backward - and the log-sum-exp
merges between them.  Prints one JSON object.

    python cp_study.py --config 5 --cp 4
    python cp_study.py --config 5 --cp 4 --all-ranks [--zigzag]
"""
import argparse
import json
import statistics
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def chunk_ranges(lengths, cp, align):
    """Per sequence the cp chunk bounds (begin, end) in local positions: boundaries on multiples
    of `align`, equal chunks of ceil(L / cp) rounded up to it, the last chunk open past L."""
    out = []
    for L in lengths:
        per = -(-int(L) // cp)
        per = max(-(-per // align) * align, align)
        out.append([(c * per, (c + 1) * per if c + 1 < cp else max(int(L), cp * per)) for c in range(cp)])
    return out


def visit_pairs(lengths, bounds, r, c):
    """Number of (query, key) pairs with key <= query inside visit (query chunk r, key chunk c)."""
    n = 0
    for L, b in zip(lengths, bounds):
        qb, qe = b[r][0], min(b[r][1], int(L))
        kb, ke = b[c][0], min(b[c][1], int(L))
        if qe <= qb or ke <= kb:
            continue
        if ke <= qb:                                   # keys strictly before the queries: a rectangle
            n += (qe - qb) * (ke - kb)
        elif kb >= qe:
            continue
        else:                                          # same chunk (the bounds never straddle otherwise)
            for i in range(max(qb, kb), qe):
                n += min(i, ke - 1) - kb + 1
    return n


def rank_visits(cid, cp, rank, reps=5, warmup=2):
    import numpy as np
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    cfg = wl.CONFIGS[cid]
    lengths = [int(l) for l in wl.seqlens(cid)]
    cu_np = wl.cu_seqlens(lengths)
    T, ml, hq, hkv, d = cfg.total_tokens, max(lengths), cfg.hq, cfg.hkv, cfg.d
    g = torch.Generator(device="cuda")
    g.manual_seed(cid)

    def rnd(h):
        return torch.randn((T, h, d), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    q, k, v, do = rnd(hq), rnd(hkv), rnd(hkv), rnd(hq)
    cu = torch.from_numpy(cu_np).cuda()
    hc = [int(x) for x in cu_np]
    ws = torch.empty(binding.workspace_bytes(T, len(lengths), hq, hkv, d, binding.HYD_BF16, 1), dtype=torch.uint8, device="cuda")
    bounds = chunk_ranges(lengths, cp, binding.RANGE_ALIGN)
    acc_o = torch.zeros_like(q)
    acc_l = torch.full((hq, T), float("-inf"), dtype=torch.float32, device="cuda")
    part_o, part_l = torch.zeros_like(q), torch.full_like(acc_l, float("-inf"))
    dq, dk, dv = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
    # the merged forward of the rank's rows, which the backward visits need
    o_full, lse_full = binding.varlen_attn_fwd(q, k, v, cu, ml, cfg.scale, cu_seqlens_host=hc)
    visits = []
    binding.enable_kernel_timing(True)
    for c in range(rank + 1):
        ranges = [(b[rank][0], b[rank][1], b[c][0], b[c][1]) for b in bounds]
        per = {}
        for it in range(warmup + reps):
            binding.varlen_attn_fwd_range(q, k, v, cu, ranges, ml, cfg.scale, part_o, part_l, cu_seqlens_host=hc, workspace=ws)
            binding.attn_merge(acc_o, acc_l, part_o, part_l, out=acc_o, lse_out=acc_l)
            binding.varlen_attn_bwd_range(q, k, v, o_full, lse_full, do, cu, ranges, ml, cfg.scale, dq, dk, dv,
                                          cu_seqlens_host=hc, workspace=ws)
            t = binding.kernel_times()
            if it >= warmup:
                for name, ms in t:
                    per.setdefault(name, []).append(ms)
        pairs = visit_pairs(lengths, bounds, rank, c)
        kms = {n: statistics.median(x) for n, x in per.items() if n != "schedule_prelude"}
        flop = {"fwd_range_bf16": 4.0, "bwd_dkdv_range_bf16": 8.0, "bwd_dq_range_bf16": 6.0}
        visits.append({"key_chunk": c, "pairs": pairs, "kernel_ms": kms,
                       "product_tflops": {n: f * d * hq * pairs / (kms[n] * 1e-3) / 1e12 for n, f in flop.items() if kms.get(n, 0) > 0}})
    binding.enable_kernel_timing(False)
    torch.cuda.synchronize()
    return {"config": cid, "cp": cp, "rank": rank, "tokens_of_rank": sum(max(0, min(b[rank][1], L) - b[rank][0]) for L, b in zip(lengths, bounds)),
            "visits": visits,
            "note": "product_tflops = matrix products the kernel performs (forward 2, dK/dV 4, dQ 3) x 2 d Hq flop x the "
                    "visible pairs of the visit / kernel time; a visit to an earlier chunk is a full rectangle (no masked work)"}


def rank_visit_list(cp, rank, zigzag):
    """(query chunk, key chunk) pairs one rank computes, and the number of chunks a sequence is cut
    into.  Contiguous: rank r owns chunk r of cp and meets chunks 0..r.  Zigzag: a sequence is cut
    into 2 cp chunks and rank r owns chunks r and 2 cp - 1 - r, which gives every rank the same
    2 cp + 1 visible (query chunk, key chunk) pairs - the usual remedy for the causal imbalance."""
    if not zigzag:
        return [(rank, c) for c in range(rank + 1)], cp
    n = 2 * cp
    mine = (rank, n - 1 - rank)
    return [(a, b) for a in mine for b in range(n) if b <= a], n


def rank_totals(cid, cp, zigzag, reps=3, warmup=1):
    """Kernel time of everything a rank computes (forward, merge, dK/dV, dQ of all its visits), for
    every rank of the CP group in turn on the one GPU."""
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    cfg = wl.CONFIGS[cid]
    lengths = [int(l) for l in wl.seqlens(cid)]
    cu_np = wl.cu_seqlens(lengths)
    T, ml, hq, hkv, d = cfg.total_tokens, max(lengths), cfg.hq, cfg.hkv, cfg.d
    g = torch.Generator(device="cuda")
    g.manual_seed(cid)

    def rnd(h):
        return torch.randn((T, h, d), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    q, k, v, do = rnd(hq), rnd(hkv), rnd(hkv), rnd(hq)
    cu = torch.from_numpy(cu_np).cuda()
    hc = [int(x) for x in cu_np]
    ws = torch.empty(binding.workspace_bytes(T, len(lengths), hq, hkv, d, binding.HYD_BF16, 1), dtype=torch.uint8, device="cuda")
    acc_o = torch.zeros_like(q)
    acc_l = torch.full((hq, T), float("-inf"), dtype=torch.float32, device="cuda")
    part_o, part_l = torch.zeros_like(q), torch.full_like(acc_l, float("-inf"))
    dq, dk, dv = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
    o_full, lse_full = binding.varlen_attn_fwd(q, k, v, cu, ml, cfg.scale, cu_seqlens_host=hc)
    out = []
    for rank in range(cp):
        visits, n_chunks = rank_visit_list(cp, rank, zigzag)
        bounds = chunk_ranges(lengths, n_chunks, binding.RANGE_ALIGN)
        ms, pairs = [], 0
        for it in range(warmup + reps):
            binding.enable_kernel_timing(True)
            for a, b in visits:
                ranges = [(x[a][0], x[a][1], x[b][0], x[b][1]) for x in bounds]
                binding.varlen_attn_fwd_range(q, k, v, cu, ranges, ml, cfg.scale, part_o, part_l, cu_seqlens_host=hc, workspace=ws)
                binding.attn_merge(acc_o, acc_l, part_o, part_l, out=acc_o, lse_out=acc_l)
                binding.varlen_attn_bwd_range(q, k, v, o_full, lse_full, do, cu, ranges, ml, cfg.scale, dq, dk, dv,
                                              cu_seqlens_host=hc, workspace=ws)
            t = binding.kernel_times()
            binding.enable_kernel_timing(False)
            if it >= warmup:
                ms.append(sum(x for n, x in t if n.endswith("range_bf16")))
        pairs = sum(visit_pairs(lengths, bounds, a, b) for a, b in visits)
        out.append({"rank": rank, "visits": len(visits), "pairs": pairs, "attention_kernel_ms": statistics.median(ms)})
    tot = [r["attention_kernel_ms"] for r in out]
    return {"config": cid, "cp": cp, "layout": "zigzag" if zigzag else "contiguous", "ranks": out,
            "max_over_mean": max(tot) / (sum(tot) / len(tot)),
            "note": "attention_kernel_ms = forward, dK/dV and dQ range kernels of all visits of the rank (merge and D passes "
                    "excluded: in this single-buffer emulation they sweep all T rows, not the rank's)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--cp", type=int, default=4)
    ap.add_argument("--rank", type=int, default=-1, help="default: the last rank, which meets every key chunk")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--all-ranks", action="store_true", help="total attention time of every rank instead of one rank's visits")
    ap.add_argument("--zigzag", action="store_true", help="with --all-ranks: rank r owns chunks r and 2cp-1-r of 2cp")
    args = ap.parse_args()
    if args.cp < 1:
        sys.exit("--cp must be at least 1")
    if args.all_ranks:
        print(json.dumps(rank_totals(args.config, args.cp, args.zigzag, max(1, args.reps // 2))))
        return
    rank = args.cp - 1 if args.rank < 0 else args.rank
    if rank >= args.cp:
        sys.exit("--rank must be below --cp")
    print(json.dumps(rank_visits(args.config, args.cp, rank, args.reps)))


if __name__ == "__main__":
    main()
