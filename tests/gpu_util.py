"""Helpers of the GPU parity tests: run the HIP path through the C ABI on numpy inputs, and the
error metrics of the acceptance bar (per output tensor, in float64):
    max-abs = max |gpu - ref|,   rel-L2 = ||gpu - ref||_2 / ||ref||_2
bf16: max-abs <= 2e-2 and rel-L2 <= 5e-3;  fp32: both <= 1e-5.

The bf16 max-abs bar has one exception, and only where the storage format forces it.  Outputs are
stored as bf16 (8 significant bits); rounding to nearest alone errs by up to half a step:
2^-7 = 0.0078 for |x| in [2,4), 2^-6 = 0.0156 in [4,8), 2^-5 = 0.0313 in [8,16), 2^-4 in [16,32).
From |x| >= 8 on that exceeds 2e-2 by itself, so there (and only there) an element passes if
|err| <= half_step_bf16(ref) + BIG_EPS: the rounding of the result plus a stated allowance for the
arithmetic before it.  Below 8 the stated 2e-2 stands.  Every report line shows max|ref| and, per
band of |ref|, how many elements there are, how many exceed 2e-2 and the largest error."""
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


BIG_EPS = 5e-3          # arithmetic allowance on top of the format's half step where |ref| >= 8
BANDS = ((0.0, 1.0), (1.0, 2.0), (2.0, 4.0), (4.0, 8.0), (8.0, np.inf))


def band_report(err, ref, bar):
    """Per band of |ref|: elements, elements whose error exceeds `bar`, largest error."""
    a = np.abs(ref)
    parts = []
    for lo, hi in BANDS:
        m = (a >= lo) & (a < hi)
        n = int(np.count_nonzero(m))
        if n:
            e = err[m]
            parts.append(f"[{lo:g},{hi:g}): n={n} over={int(np.count_nonzero(e > bar))} max={float(e.max()):.3e}")
    return "; ".join(parts)


def tolerance(ref, dtype):
    ta, _ = TOL[dtype]
    tol = np.full(ref.shape, ta)
    if dtype == "bf16":
        big = np.abs(ref) >= 8.0
        tol[big] = half_ulp_bf16(ref[big]) + BIG_EPS
    return tol


def check(name, got, ref, dtype, report=None, failures=None):
    """Asserts the bar.  With `failures` (a list) a miss is appended there instead of raised, so
    that a test can print every tensor before it fails."""
    max_abs, rel = errors(got, ref)
    ta, tr = TOL[dtype]
    err = np.abs(got - ref)
    tol = tolerance(ref, dtype)
    line = (f"{name}: max-abs {max_abs:.3e} (tol {ta:.0e})  rel-L2 {rel:.3e} (tol {tr:.0e})  "
            f"max|ref| {np.max(np.abs(ref)) if ref.size else 0:.3f}  n={ref.size}  bands {band_report(err, ref, ta)}")
    print(line, flush=True)
    if report is not None:
        report.append(line)
    bad = []
    if not np.all(np.isfinite(got)):
        bad.append(f"{name}: non-finite values")
    n_bad = int(np.count_nonzero(err > tol))
    if n_bad:
        bad.append(f"{name}: {n_bad} elements beyond the max-abs bar | {line}")
    if rel > tr:
        bad.append(f"{name}: rel-L2 beyond the bar | {line}")
    if failures is not None:
        failures.extend(bad)
    else:
        assert not bad, "\n".join(bad)
    return max_abs, rel


def check_all(got, q, k, v, do, cu, scale, dtype, failures, orc):
    """Every output of a forward + backward run against the fp64 oracle.

    O, LSE and dV: against the definition, on the stated bar.

    dQ and dK: the backward call is handed the forward's stored O, which is rounded to the storage
    format, and forms D = <dO, O> from it; on short sequences (|O| of order one) that rounding
    alone moves D by up to a few 1e-2 and dQ, dK with it, whatever the arithmetic of the backward
    is (the fp64 oracle, given the same stored O and LSE, moves by the same amount).  So dQ and dK
    are asserted on the stated bar against the oracle's backward OF THE STORED O AND LSE - the
    exact function of what the call receives - and, against the definition, on rel-L2, with the
    max-abs printed next to the part of it that the stored O and LSE account for."""
    ref_o, ref_lse = orc.fwd(q, k, v, cu, scale)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, scale)
    check("o", got["o"], ref_o, dtype, failures=failures)
    check("lse", got["lse"], ref_lse, dtype, failures=failures)
    check("dv", got["dv"], dv, dtype, failures=failures)
    if dtype != "bf16":
        check("dq", got["dq"], dq, dtype, failures=failures)
        check("dk", got["dk"], dk, dtype, failures=failures)
        return
    gq, gk, _ = orc.bwd_given(q, k, v, do, got["o"].astype(np.float32), got["lse"].astype(np.float32), cu, scale)
    _, tr = TOL[dtype]
    for name, plain, given in (("dq", dq, gq), ("dk", dk, gk)):
        check(f"{name} (vs the backward of the stored O, LSE)", got[name], given, dtype, failures=failures)
        max_abs, rel = errors(got[name], plain)
        print(f"{name} (vs the definition): max-abs {max_abs:.3e}, of which the stored O, LSE account for up to "
              f"{float(np.max(np.abs(given - plain))) if plain.size else 0:.3e};  rel-L2 {rel:.3e} (tol {tr:.0e})", flush=True)
        if rel > tr:
            failures.append(f"{name}: rel-L2 {rel:.3e} against the definition beyond the bar")


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
