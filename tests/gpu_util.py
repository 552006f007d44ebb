"""Helpers of the GPU parity tests: run the HIP path through the C ABI on numpy inputs, and the
error metrics of the acceptance bar (per output tensor, in float64):
    max-abs = max |gpu - ref|,   rel-L2 = ||gpu - ref||_2 / ||ref||_2
bf16: max-abs <= 2e-2 and rel-L2 <= 5e-3;  fp32: both <= 1e-5.

The bf16 max-abs bar needs one derived exception.  Outputs are stored as bf16, and rounding to
nearest alone errs by up to half an ulp: 2^-7 for |x| in [4,8), 2^-6 in [8,16), 2^-5 in [16,32).
From |x| >= 8 on that exceeds 2e-2 by itself, and in [4,8) it leaves the arithmetic only 4e-3.
So an element passes if |err| <= max(2e-2, half_ulp_bf16(ref) + 1e-2): the stated 2e-2 wherever
the format allows it (|ref| < 4), and "format rounding plus 1e-2 of arithmetic error" above.
Every report line also shows max|ref| and how many elements needed the exception."""
import numpy as np
import torch

from paper_2412_07894_amd import binding, workloads as wl

TOL = {"bf16": (2e-2, 5e-3), "fp32": (1e-5, 1e-5)}


def to_dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t       # values are bf16-exact already


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def run_gpu(cu, q, k, v, do, dtype, scale, host_cu=True, o_lse=None):
    """Forward then backward on the GPU; the backward consumes the GPU forward's own O and LSE
    (the training dataflow) unless o_lse=(O, LSE) numpy arrays are given."""
    cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    lens = np.diff(cu)
    max_len = int(lens.max()) if len(lens) else 0
    qd, kd, vd, dod = (to_dev(x, dtype) for x in (q, k, v, do))
    hc = [int(x) for x in cu] if host_cu else None
    o, lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, max_len, scale, cu_seqlens_host=hc)
    if o_lse is not None:
        o_in, lse_in = to_dev(o_lse[0].astype(np.float32), dtype), torch.from_numpy(o_lse[1].astype(np.float32)).cuda()
    else:
        o_in, lse_in = o, lse
    dq, dk, dv = binding.varlen_attn_bwd(qd, kd, vd, o_in, lse_in, dod, cu_d, max_len, scale, cu_seqlens_host=hc)
    torch.cuda.synchronize()
    return {"o": to_np(o), "lse": to_np(lse), "dq": to_np(dq), "dk": to_np(dk), "dv": to_np(dv)}


def errors(got, ref):
    diff = got - ref
    denom = float(np.sqrt((ref * ref).sum()))
    return float(np.max(np.abs(diff))) if diff.size else 0.0, (float(np.sqrt((diff * diff).sum())) / denom if denom > 0 else 0.0)


def half_ulp_bf16(x):
    """Half the spacing of bfloat16 (8 significant bits) at |x|."""
    a = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 8)


def check(name, got, ref, dtype, report=None):
    max_abs, rel = errors(got, ref)
    ta, tr = TOL[dtype]
    err = np.abs(got - ref)
    tol = np.full(ref.shape, ta)
    if dtype == "bf16":
        tol = np.maximum(tol, half_ulp_bf16(ref) + 1e-2)
    n_exc = int(np.count_nonzero(err > ta))
    line = (f"{name}: max-abs {max_abs:.3e} (tol {ta:.0e})  rel-L2 {rel:.3e} (tol {tr:.0e})  "
            f"max|ref| {np.max(np.abs(ref)) if ref.size else 0:.3f}  elements over {ta:.0e} (format-limited): {n_exc}")
    print(line, flush=True)
    if report is not None:
        report.append(line)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    assert np.all(err <= tol), line
    assert rel <= tr, line


def sample_rows(cu, hq, rng, n_random):
    """Sampled (token, head) pairs for full-size checks: sequence starts and ends, tile boundaries,
    the longest and the shortest sequence, plus n_random uniform draws."""
    lens = np.diff(cu)
    toks = []
    longest = int(np.argmax(lens))
    for s in {0, longest, len(lens) - 1, int(np.argmin(np.where(lens > 0, lens, 1 << 30)))}:
        a, L = int(cu[s]), int(lens[s])
        for off in (0, 1, 31, 32, 63, 64, 127, 128, 255, 256, L // 2, L - 2, L - 1):
            if 0 <= off < L:
                toks.append(a + off)
    toks += [int(t) for t in rng.integers(0, int(cu[-1]), n_random)]
    toks = np.array(sorted(set(toks)), dtype=np.int32)
    heads = rng.integers(0, hq, len(toks)).astype(np.int32)
    return toks, heads
