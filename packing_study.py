#!/usr/bin/env python3
"""Cost-aware packing measured on this library's own kernels (Hydraulis, arXiv 2412.07894,
Sec. 6.1 and App. C.2, D): fit T(l) = a l^2 + b l + c to the measured forward+backward time of
sequences inside packed buffers, pack a length draw into micro-batches once the way the paper argues against
(fill to the maximum length, first fit decreasing) and once by Eq. 1 (minimise the longest
micro-batch times (PP - 1 + V), V enumerated), then run every micro-batch of both packings on the
GPU and compare predicted with measured times.  With --dispatch the draw is first dispatched over
four simulated pipelines (Sec. 6.2, Alg. 1 against length buckets).  Prints one JSON object.

    python packing_study.py --config 5 --pp 4
    python packing_study.py --config 3 --pp 4 --dispatch
"""
import argparse
import json
import statistics
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def time_lengths(lengths, hq, hkv, d, reps, warmup, seed=0):
    """Median milliseconds of one forward + backward over one packed buffer holding `lengths`."""
    import numpy as np
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    cu_np = wl.cu_seqlens(lengths)
    T, ml = int(cu_np[-1]), int(max(lengths))
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)

    def rnd(h):
        return torch.randn((T, h, d), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    q, k, v, do = rnd(hq), rnd(hkv), rnd(hkv), rnd(hq)
    cu = torch.from_numpy(cu_np).cuda()
    scale = 1.0 / float(np.sqrt(d))
    ws_f = torch.empty(binding.workspace_bytes(T, len(lengths), hq, hkv, d, binding.HYD_BF16, 0), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(binding.workspace_bytes(T, len(lengths), hq, hkv, d, binding.HYD_BF16, 1), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty((hq, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ms = []
    for it in range(warmup + reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        binding.varlen_attn_fwd(q, k, v, cu, ml, scale, workspace=ws_f, out=o, lse=lse)
        binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, scale, workspace=ws_b, dq=dq, dk=dk, dv=dv)
        e1.record()
        e1.synchronize()
        if it >= warmup:
            ms.append(e0.elapsed_time(e1))
    return statistics.median(ms)


def calibrate(hq, hkv, d, probe_lengths, cap, reps=5, warmup=2):
    """Profiled (length, ms) points and the model fitted to them (App. C.2).  The time of a
    sequence of length l is taken inside a packed buffer, as it will run: a buffer of
    k = cap // l copies is timed and divided by k, so that what is paid once per call (launches,
    the schedule prelude) is not charged to every sequence."""
    from paper_2412_07894_amd import planner
    times = []
    for l in probe_lengths:
        k = max(1, int(cap) // int(l))
        times.append(time_lengths([int(l)] * k, hq, hkv, d, reps, warmup, seed=int(l)) / k)
    # relative errors (weights 1 / t^2): the times span three orders of magnitude
    model = planner.fit_latency([float(l) for l in probe_lengths], times, [1.0 / (t * t) for t in times])
    return model, times


def util_len(model, max_len, threshold=0.85):
    """Length from which the per-token cost that packing can amortise (b + c/l, the part of
    T(l)/l that does not grow with l) is within 1/threshold of its floor b: the reading of
    App. D's "efficiency reaches a threshold (0.85)" for a model that prices attention only."""
    a, b, c = model.as_tuple()
    if b <= 0 or c <= 0:
        return 1
    return int(max(1, min(max_len, round(c / (b * (1.0 / threshold - 1.0))))))


def study(lengths, hq, hkv, d, max_len, pp, probe_lengths, reps=5, warmup=2, node_limit=2_000_000):
    from paper_2412_07894_amd import planner
    model, probe_ms = calibrate(hq, hkv, d, probe_lengths, max_len, reps, warmup)
    # what one call costs before any sequence does: launches and the schedule prelude.  Eq. 1 does
    # not price it (its T(l) is per sequence); it is added to the predictions below so that they
    # can be compared with measured micro-batch times.
    call_ms = time_lengths([64], hq, hkv, d, reps, warmup)
    ul = util_len(model, max_len)
    out = {"heads": [hq, hkv], "head_dim": d, "max_len": max_len, "pp": pp, "num_seqs": len(lengths),
           "tokens": int(sum(lengths)), "model_ms": dict(zip("abc", model.as_tuple())),
           "probe": {"lengths": [int(l) for l in probe_lengths], "ms": probe_ms,
                     "fit_rel_err": [abs(planner.latency(model, l) - t) / t for l, t in zip(probe_lengths, probe_ms)]},
           "call_overhead_ms": call_ms, "util_len": ul, "v_range": list(planner.v_range(lengths, max_len, ul))}
    v_ffd, a_ffd = planner.pack_ffd(lengths, max_len)
    obj, v_bal, a_bal, proven = planner.pack(lengths, model, max_len, ul, pp, node_limit)
    for name, V, assign in (("max_length_ffd", v_ffd, a_ffd), ("balanced_eq1", v_bal, a_bal)):
        batches = [[int(l) for l, j in zip(lengths, assign) if j == b] for b in range(V)]
        pred = [call_ms + sum(planner.latency(model, l) for l in mb) for mb in batches]
        meas = [time_lengths(mb, hq, hkv, d, reps, warmup, seed=17 + b) for b, mb in enumerate(batches)]
        out[name] = {
            "V": V, "tokens_per_batch": [sum(mb) for mb in batches], "seqs_per_batch": [len(mb) for mb in batches],
            "predicted_ms": pred, "measured_ms": meas,
            "predicted_objective_ms": max(pred) * (pp - 1 + V), "measured_objective_ms": max(meas) * (pp - 1 + V),
            "measured_sum_ms": sum(meas), "measured_max_over_mean": max(meas) / (sum(meas) / V),
        }
    out["balanced_eq1"]["search_finished"] = proven
    out["measured_objective_ratio_ffd_over_balanced"] = (
        out["max_length_ffd"]["measured_objective_ms"] / out["balanced_eq1"]["measured_objective_ms"])
    return out


def dispatch_study(lengths, hq, hkv, d, max_lens, pps, trials, probe_lengths, reps=5, warmup=2, seed=0,
                   node_limit=500_000):
    """Sec. 6.2 on one GPU: the D pipelines are simulated one after the other with the same
    kernels (one latency model), and differ in the longest sequence they admit and in depth.
    Dispatches a mini-batch once by Alg. 1 and once by length buckets (every sequence to the
    tightest pipeline that admits it: the naive approach of Sec. 6.2), packs each pipeline's share
    by Eq. 1, runs every micro-batch and prices a pipeline at max micro-batch time x (PP-1+V)."""
    import random
    from paper_2412_07894_amd import planner
    D = len(max_lens)
    assert all(max_lens[j] >= max_lens[j + 1] for j in range(D - 1))
    model, probe_ms = calibrate(hq, hkv, d, probe_lengths, max_lens[0], reps, warmup)
    call_ms = time_lengths([64], hq, hkv, d, reps, warmup)
    J = [sum(1 for m in max_lens if m >= l) for l in lengths]
    rng = random.Random(seed)
    perms = [rng.sample(range(len(lengths)), len(lengths)) for _ in range(trials)]
    cost, greedy = planner.dispatch(lengths, J, [model] * D, pps, perms)
    buckets = [j - 1 for j in J]
    out = {"heads": [hq, hkv], "max_lens": list(max_lens), "pps": list(pps), "trials": trials,
           "num_seqs": len(lengths), "tokens": int(sum(lengths)), "model_ms": dict(zip("abc", model.as_tuple())),
           "call_overhead_ms": call_ms, "greedy_cost_bound_ms": cost}
    for name, assign in (("length_buckets", buckets), ("greedy_alg1", greedy)):
        pipes = []
        for j in range(D):
            mine = [int(l) for l, p in zip(lengths, assign) if p == j]
            if not mine:
                pipes.append({"seqs": 0, "tokens": 0, "V": 0, "bound_ms": 0.0, "measured_ms": 0.0})
                continue
            bound = sum(planner.latency(model, l) for l in mine) + planner.latency(model, max(mine)) * (pps[j] - 1)
            _, V, a, _ = planner.pack(mine, model, max_lens[j], util_len(model, max_lens[j]), pps[j], node_limit)
            batches = [[l for l, b in zip(mine, a) if b == k] for k in range(V)]
            meas = [time_lengths(mb, hq, hkv, d, reps, warmup, seed=31 * j + k) for k, mb in enumerate(batches)]
            pipes.append({"seqs": len(mine), "tokens": sum(mine), "V": V, "bound_ms": bound,
                          "measured_ms": max(meas) * (pps[j] - 1 + V), "micro_batch_ms": meas})
        out[name] = {"pipelines": pipes, "max_bound_ms": max(p["bound_ms"] for p in pipes),
                     "max_measured_ms": max(p["measured_ms"] for p in pipes)}
    out["measured_ratio_buckets_over_greedy"] = out["length_buckets"]["max_measured_ms"] / out["greedy_alg1"]["max_measured_ms"]
    return out


def main():
    from paper_2412_07894_amd import workloads as wl
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=5, choices=[2, 3, 4, 5])
    ap.add_argument("--pp", type=int, default=4)
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--dispatch", action="store_true",
                    help="dispatch the draw over 4 simulated pipelines (Sec. 6.2) instead of packing one")
    args = ap.parse_args()
    cfg = wl.CONFIGS[args.config]
    lengths = [int(l) for l in wl.seqlens(args.config)]
    probes = [l for l in (256, 512, 1024, 2048, 4096, 8192, 12288, 16384, 24576, 32768, 49152, 65536)
              if l <= cfg.buffer_tokens]
    if args.dispatch:
        cap = cfg.buffer_tokens
        res = dispatch_study(lengths, cfg.hq, cfg.hkv, cfg.d, [cap, cap // 2, cap // 4, cap // 4],
                             [args.pp, args.pp, 2, 2], 100, probes, reps=args.reps)
        res["workload"] = f"config {cfg.cid}: {cfg.name}"
        print(json.dumps(res))
        return 0
    res = study(lengths, cfg.hq, cfg.hkv, cfg.d, cfg.buffer_tokens, args.pp, probes, reps=args.reps)
    res["workload"] = f"config {cfg.cid}: {cfg.name}"
    print(json.dumps(res))


if __name__ == "__main__":
    sys.exit(main())
