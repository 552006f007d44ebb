#!/usr/bin/env python3
"""Benchmark of the hot path: packed varlen causal attention, forward + backward, on one MI355X.

One "step" is one forward call plus one backward call (schedule preludes, forward kernel, row
statistics and fp16 operand copies, dK/dV kernel, dQ kernel) over one synthetic packed batch that
is already resident in HBM.  By default the four bf16 configurations of the benchmark spec (2-5) are
timed one after the other, each for `--steps` steps after `--warmup` warm-up steps, and the
headline is the SLOWEST of them (lowest useful TFLOP/s); `--config N` times one configuration
only (this is what the rocprofv3 runs under profiles/ use).  Prints ONE JSON line:
    value        useful causal TFLOP/s = 14 * d * Hq * sum_s L_s (L_s + 1) / 2 / step time of the
                 headline configuration; `all_configs` holds the same figures for every one timed
    roofline     the dominant kernel (dK/dV) of the headline configuration against the bf16/fp16
                 dense MFMA peak, its duration measured with HIP events on the launch stream inside
                 the timed region
    cpu_baseline the fp64 oracle timed on this host's cores on a bounded sample of the workload
    mfma_probe   what a loop of nothing but bf16 MFMAs sustains on this board, with all-zero and
                 with random operands (outside the timed region, from the bench-only helper
                 bench_probe.so): the board lowers its clock when operand bits toggle, so the
                 nominal peak is not what real data can reach
`--inputs zeros` runs the same kernels on all-zero tensors (a diagnostic of that same effect,
never the headline number).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0           # MI355X dense bf16 MFMA


def gpu_inputs(cfg, lengths, seed, inputs="randn"):
    import torch
    from paper_2412_07894_amd import workloads as wl
    T = cfg.total_tokens
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)

    def rnd(h):
        if inputs == "zeros":
            return torch.zeros((T, h, cfg.d), device="cuda", dtype=dt)
        return torch.randn((T, h, cfg.d), device="cuda", dtype=torch.float32, generator=g).to(dt)
    cu = torch.from_numpy(wl.cu_seqlens(lengths)).cuda()
    return rnd(cfg.hq), rnd(cfg.hkv), rnd(cfg.hkv), rnd(cfg.hq), cu


def mfma_probe():
    """Sustained TFLOP/s of a pure bf16 MFMA loop and of the forward tile's instruction mix (about 15 ms per
    launch), zeros and random operands; None when the helper library has not been built."""
    import ctypes
    import torch
    path = os.path.join(ROOT, "bench_probe.so")
    if not os.path.exists(path):
        return None
    lib = ctypes.CDLL(path)
    lib.bench_probe_mfma.restype = ctypes.c_int
    lib.bench_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                     ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float)]
    out = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    res = {}
    for name, pattern, iters in (("zeros", 0, 100000), ("random", 1, 100000), ("fwd_mix_zeros", 2, 20000), ("fwd_mix_random", 3, 20000)):
        best = 0.0
        for _ in range(3):
            flops, ms = ctypes.c_double(0.0), ctypes.c_float(0.0)
            if lib.bench_probe_mfma(256, iters, pattern, out.data_ptr(), ctypes.byref(flops), ctypes.byref(ms)) != 0:
                return None
            best = max(best, flops.value / (ms.value * 1e-3) / 1e12)
        res[name] = best
    res["unit"] = "TFLOP/s"
    res["what"] = ("256 workgroups x 8 waves of v_mfma_f32_32x32x16_bf16 on register operands, best of 3 launches; "
                   "fwd_mix_*: the same MFMAs inside the forward tile's instruction mix (one LDS fragment per MFMA, the "
                   "softmax arithmetic of one score per MFMA), no synchronisation")
    return res


def run_gpu(cid, steps, warmup, inputs="randn"):
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    cfg = wl.CONFIGS[cid]
    lengths = wl.seqlens(cid)
    q, k, v, do, cu = gpu_inputs(cfg, lengths, seed=1000 * cid, inputs=inputs)
    T, nseq, ml = cfg.total_tokens, len(lengths), int(max(lengths))
    code = binding.HYD_BF16 if cfg.dtype == "bf16" else binding.HYD_FP32
    ws_f = torch.empty(binding.workspace_bytes(T, nseq, cfg.hq, cfg.hkv, cfg.d, code, 0), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(binding.workspace_bytes(T, nseq, cfg.hq, cfg.hkv, cfg.d, code, 1), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty((cfg.hq, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    per_kernel = {}

    def step():
        binding.varlen_attn_fwd(q, k, v, cu, ml, cfg.scale, workspace=ws_f, out=o, lse=lse)
        binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, cfg.scale, workspace=ws_b, dq=dq, dk=dk, dv=dv)

    # one plain copy kernel of known size (256 MiB read, 256 MiB written), outside the timed
    # region: the reference that scales the HBM counters of a `rocprofv3 --pmc` run of this command
    cal = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    torch.add(cal, 0.0, out=torch.empty_like(cal))
    del cal
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps; the library brackets every kernel with HIP events on
    # the launch stream and only records them: the events are read after the region has ended
    binding.enable_kernel_timing(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    recorded = binding.kernel_times()
    for name, ms in recorded:
        per_kernel.setdefault(name, []).append(ms)
    binding.enable_kernel_timing(False)
    # kernel time of each step (the recorded launches split evenly over the steps): mean, std, min
    per_step = []
    if recorded and len(recorded) % steps == 0:
        n = len(recorded) // steps
        per_step = [sum(ms for _, ms in recorded[i * n:(i + 1) * n]) for i in range(steps)]
    ms_per_step = (t1 - t0) * 1e3 / steps
    pairs = wl.causal_pairs(lengths)
    # per launch; the schedule prelude runs twice per step (forward; backward: one launch builds the lists of dK/dV and dQ)
    kernels = {n: sum(x) / len(x) for n, x in per_kernel.items()}
    return cfg, lengths, pairs, ms_per_step, kernels, per_step


def per_buffer(cid, reps=5, warmup=2):
    """The paper's micro-batch view (Sec. 2.1, Fig. 2): one forward+backward call per packed buffer
    of the configuration, one after the other; equal token counts, very different times."""
    import statistics
    import numpy as np
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    cfg = wl.CONFIGS[cid]

    def time_lengths(lens, seed):
        """Median milliseconds of one forward + backward over one packed buffer holding `lens`."""
        T, ml = int(sum(lens)), int(max(lens))
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        rnd = lambda h: torch.randn((T, h, cfg.d), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
        q, k, v, do = rnd(cfg.hq), rnd(cfg.hkv), rnd(cfg.hkv), rnd(cfg.hq)
        cu = torch.from_numpy(wl.cu_seqlens(lens)).cuda()
        ms = []
        for it in range(warmup + reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            o, lse = binding.varlen_attn_fwd(q, k, v, cu, ml, cfg.scale)
            binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, cfg.scale)
            e1.record()
            torch.cuda.synchronize()
            if it >= warmup:
                ms.append(e0.elapsed_time(e1))
        return statistics.median(ms)

    lengths = [int(l) for l in wl.seqlens(cid)]
    buffers, cur = [], []
    for l in lengths:                       # buffers are exactly full and listed one after the other
        cur.append(l)
        if sum(cur) == cfg.buffer_tokens:
            buffers.append(cur)
            cur = []
    if cur or len(buffers) != cfg.n_buffers:
        return None
    ms = [time_lengths(b, seed=i) for i, b in enumerate(buffers)]
    tf = [14.0 * cfg.d * cfg.hq * wl.causal_pairs(b) / 1e12 for b in buffers]
    return {"tokens_per_buffer": cfg.buffer_tokens, "seqs": [len(b) for b in buffers], "longest": [max(b) for b in buffers],
            "ms": ms, "useful_tflop": tf, "max_over_min_ms": max(ms) / min(ms), "sum_ms": sum(ms)}


def rope_study(cid, reps=10, warmup=3):
    """Position reset for Q (Sec. 2.1): the rotary embedding of Q applied inside the kernels
    (hyd_varlen_attn_fwd_rope / _bwd_rope) against passes of their own over Q and dQ
    (hyd_rope_packed before the forward, its inverse after the backward).  K is rotated by its own
    pass either way and is not timed.  Median milliseconds of one forward + backward."""
    import statistics
    import torch
    from paper_2412_07894_amd import binding, workloads as wl
    cfg = wl.CONFIGS[cid]
    lengths = wl.seqlens(cid)
    q, k, v, do, cu = gpu_inputs(cfg, lengths, seed=1000 * cid)
    ml = int(max(lengths))
    q_rot, dq_un = torch.empty_like(q), torch.empty_like(q)

    def timed(fn):
        ms = []
        for it in range(warmup + reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            if it >= warmup:
                ms.append(e0.elapsed_time(e1))
        return statistics.median(ms)

    def fused():
        o, lse = binding.varlen_attn_fwd(q, k, v, cu, ml, cfg.scale, rope_base=10000.0)
        binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, cfg.scale, rope_base=10000.0)

    def separate():
        binding.rope_packed(q, cu, out=q_rot)
        o, lse = binding.varlen_attn_fwd(q_rot, k, v, cu, ml, cfg.scale)
        dq, _, _ = binding.varlen_attn_bwd(q_rot, k, v, o, lse, do, cu, ml, cfg.scale)
        binding.rope_packed(dq, cu, inverse=True, out=dq_un)

    def plain():
        o, lse = binding.varlen_attn_fwd(q, k, v, cu, ml, cfg.scale)
        binding.varlen_attn_bwd(q, k, v, o, lse, do, cu, ml, cfg.scale)

    return {"config": cid, "ms_no_rotation": timed(plain), "ms_rotation_inside_the_kernels": timed(fused),
            "ms_rotation_by_two_passes_over_q_and_dq": timed(separate)}


def cpu_baseline(cid):
    """The fp64 oracle, as it stands, on a bounded sample of the workload (about 2-3e12 flop,
    10-30 s on 16 cores): as many KV groups as the oracle has threads (its OpenMP loop runs over
    (sequence, KV group) units), and the sequences of the configuration from the shortest up
    until the budget is spent; forward + backward."""
    from oracle import attn_oracle as orc
    from paper_2412_07894_amd import workloads as wl
    cfg = wl.CONFIGS[cid]
    lengths = wl.seqlens(cid)
    G = cfg.hq // cfg.hkv
    groups = int(max(1, min(cfg.hkv, orc.threads())))
    budget = 3.0e12 / groups
    sample, spent = [], 0.0
    for L in sorted(lengths):
        cost = 14.0 * cfg.d * G * (L * (L + 1) // 2)
        if sample and spent + cost > budget:
            break
        sample.append(L)
        spent += cost
    per_group = 14.0 * cfg.d * G * wl.causal_pairs(sample)
    cu, q, k, v, do = wl.custom(sample, groups * G, groups, cfg.d, cfg.dtype, seed=77)
    t0 = time.perf_counter()
    orc.fwd(q, k, v, cu, cfg.scale)
    orc.bwd(q, k, v, do, cu, cfg.scale)
    dt = time.perf_counter() - t0
    flops = per_group * groups
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.threads(), "kind": "oracle",
        "sample": f"fp64 oracle fwd+bwd on the {len(sample)} shortest of the {len(lengths)} sequences of config {cid} "
                  f"({int(sum(sample))} of {cfg.total_tokens} tokens, longest {max(sample)}), {groups * G} of {cfg.hq} "
                  f"query heads ({groups} KV groups), {flops / 1e12:.2f} useful TFLOP in {dt:.1f} s",
    }


def measured_traffic(cid, kernel):
    """Scaled HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary
    (profiles/hbm_traffic_summary.txt), or None when no counter run covers this workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_summary.txt")
    try:
        for line in open(path):
            parts = [x.strip() for x in line.split("|")]
            if len(parts) == 3 and parts[0] == f"config {cid}" and parts[1] == kernel:
                return float(parts[2])
    except OSError:
        pass
    return None


def config_result(cid, steps, warmup, inputs):
    """Times one configuration and returns its figures (value, ms per step, kernels, roofline)."""
    import statistics
    cfg, lengths, pairs, ms_per_step, kernels, per_step = run_gpu(cid, steps, warmup, inputs)
    useful = 14.0 * cfg.d * cfg.hq * pairs
    value = useful / (ms_per_step * 1e-3) / 1e12
    res = {
        "cid": cfg.cid, "dtype": cfg.dtype, "value": value, "ms_per_step": ms_per_step,
        "pct_of_bf16_mfma_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "config": {"workload": f"config {cfg.cid}: {cfg.name}", "total_tokens": cfg.total_tokens,
                   "num_seqs": len(lengths), "max_seqlen": int(max(lengths)), "hq": cfg.hq, "hkv": cfg.hkv,
                   "head_dim": cfg.d, "causal_pairs": pairs, "useful_flop_per_step": useful},
        "kernel_ms": kernels,
    }
    if per_step:
        res["kernel_ms_per_step"] = {"mean": statistics.fmean(per_step), "std": statistics.pstdev(per_step), "min": min(per_step),
                                     "what": "sum of the HIP-event durations of one step's kernels (launch gaps excluded)"}
    # dominant kernel: dK/dV.  Algorithmic work = the three products only it provides
    # (dV = P^T dO, dP = dO V^T, dK = dS^T Q): 6 * d * Hq flop per causal pair.
    dom = "bwd_dkdv_bf16" if cfg.dtype == "bf16" else "bwd_dkdv_fp32"
    if dom in kernels and kernels[dom] > 0:
        alg = 6.0 * cfg.d * cfg.hq * pairs
        ach = alg / (kernels[dom] * 1e-3) / 1e12
        peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else 157.3
        res["roofline"] = {"kernel": dom, "bound": "mfma" if cfg.dtype == "bf16" else "alu", "achieved": ach,
                           "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "traffic": measured_traffic(cfg.cid, dom),
                           "avg_ms": kernels[dom]}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="0 (default): configurations 2-5, headline = the slowest; N: only configuration N")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-probe", action="store_true")
    ap.add_argument("--inputs", default="randn", choices=["randn", "zeros"])
    ap.add_argument("--per-buffer", action="store_true", help="also time one call per packed buffer")
    ap.add_argument("--rope-study", action="store_true", help="also time the rotary embedding of Q inside the kernels against passes of its own")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a single-GPU hot path (no collectives, no sharding); run with --gpus 1")

    cids = [2, 3, 4, 5] if args.config == 0 else [args.config]
    t_all = time.perf_counter()
    results = [config_result(c, args.steps, args.warmup, args.inputs) for c in cids]
    wall = time.perf_counter() - t_all
    head = min(results, key=lambda r: r["value"])
    out = {
        "metric": "packed varlen attn fwd+bwd useful TFLOP/s + % of bf16 MFMA peak, 1 GPU",
        "value": head["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic" if args.inputs == "randn" else "synthetic (all-zero tensors: diagnostic only)",
        "pct_of_bf16_mfma_peak": head["pct_of_bf16_mfma_peak"],
        "config": head["config"],
        "kernel_ms": head["kernel_ms"],
    }
    if len(results) > 1:
        out["headline_rule"] = (f"configurations {cids} timed one after the other, {args.steps} steps each after {args.warmup} "
                                "warm-up steps; value is the lowest of them")
        out["all_configs"] = {f"config {r['cid']}": {k: r[k] for k in ("value", "ms_per_step", "pct_of_bf16_mfma_peak", "kernel_ms", "roofline") if k in r}
                              for r in results}
        out["all_configs_wall_s"] = wall
    for key in ("kernel_ms_per_step", "roofline"):
        if key in head:
            out[key] = head[key]
    if not args.no_mfma_probe and head["dtype"] == "bf16":
        probe = mfma_probe()
        if probe is not None:
            out["mfma_probe"] = probe
    if args.per_buffer and head["dtype"] == "bf16":
        out["per_buffer"] = per_buffer(head["cid"])
    if args.rope_study and head["dtype"] == "bf16":
        out["rope_study"] = [rope_study(r["cid"]) for r in results if r["dtype"] == "bf16"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(head["cid"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
