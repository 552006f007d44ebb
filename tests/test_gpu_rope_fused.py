"""Rotary embedding of Q inside the attention kernels (hyd_varlen_attn_fwd_rope / _bwd_rope)
against the composition of the two fp64 references: attention of (rotated Q, rotated K, V), and
the gradient of the UNROTATED Q, which is the inverse rotation of the gradient of the rotated Q.
K is rotated on the host in fp64 and rounded to bf16 once; both sides get those same bytes."""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from oracle import rope_oracle as ro
from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def round_bf16(x):
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32)))


def run_case(lengths, hq, hkv, d, seed, base):
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", seed)
    scale = 1.0 / float(np.sqrt(d))
    k_rot = round_bf16(ro.rope_packed(k, cu, base=base))                 # what a rotary pass over K leaves in HBM
    q_rot = round_bf16(ro.rope_packed(q, cu, base=base))                 # never stored; the kernels round it to bf16 as a pass of its own would
    print(f"\nfused rotary: lengths={lengths[:10]} hq={hq} hkv={hkv} d={d} base={base}", flush=True)
    cu_d = torch.from_numpy(cu).cuda()
    qd, kd, vd, dod = (gu.to_dev(x, "bf16") for x in (q, k_rot, v, do))
    hc = [int(x) for x in cu]
    o, lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, max(lengths), scale, cu_seqlens_host=hc, rope_base=base)
    dq, dk, dv = binding.varlen_attn_bwd(qd, kd, vd, o, lse, dod, cu_d, max(lengths), scale, cu_seqlens_host=hc, rope_base=base)
    torch.cuda.synchronize()
    got = {"o": gu.to_np(o), "lse": gu.to_np(lse), "dq": gu.to_np(dq), "dk": gu.to_np(dk), "dv": gu.to_np(dv)}
    q_rot32 = q_rot.astype(np.float32)
    ref_o, ref_lse = orc.fwd(q_rot32, k_rot, v, cu, scale)
    _, _, ref_dv = orc.bwd(q_rot32, k_rot, v, do, cu, scale)
    gq_rot, gk, _ = orc.bwd_given(q_rot32, k_rot, v, do, got["o"].astype(np.float32), got["lse"].astype(np.float32), cu, scale)
    ref_dq = ro.rope_packed(gq_rot, cu, base=base, inverse=True)          # gradient of the unrotated Q
    failures = []
    gu.check("o", got["o"], ref_o, "bf16", failures=failures)
    gu.check("lse", got["lse"], ref_lse, "bf16", failures=failures)
    gu.check("dv", got["dv"], ref_dv, "bf16", failures=failures)
    gu.check("dq (unrotated Q; vs the backward of the stored O, LSE)", got["dq"], ref_dq, "bf16", failures=failures)
    gu.check("dk (rotated K; vs the backward of the stored O, LSE)", got["dk"], gk, "bf16", failures=failures)
    assert not failures, "\n".join(failures)
    return got, (qd, kd, vd, dod, cu_d, hc, scale)


@pytest.mark.parametrize("lengths,hq,hkv,d,base", [
    ([1, 7, 64, 184, 0, 33], 4, 2, 128, 10000.0),
    ([513, 300], 2, 1, 128, 500000.0),
    ([700, 129], 4, 4, 64, 10000.0),
])
def test_fused_rotary_matches_the_composed_references(lengths, hq, hkv, d, base):
    run_case(lengths, hq, hkv, d, seed=61, base=base)


def test_fused_rotary_equals_rotating_q_first():
    """The same forward with Q rotated by the stand-alone kernel first: both paths round the
    rotated Q to bf16, so O and LSE agree up to the rare element whose rotation rounds the other
    way (the two kernels form their cosines differently)."""
    lengths, hq, hkv, d, base = [1500, 260], 4, 2, 128, 10000.0
    got, (qd, kd, vd, dod, cu_d, hc, scale) = run_case(lengths, hq, hkv, d, seed=62, base=base)
    q_rot_d = binding.rope_packed(qd, cu_d, base=base)
    o2, lse2 = binding.varlen_attn_fwd(q_rot_d, kd, vd, cu_d, max(lengths), scale, cu_seqlens_host=hc)
    torch.cuda.synchronize()
    assert np.max(np.abs(gu.to_np(o2) - got["o"])) <= 2e-2 and np.max(np.abs(gu.to_np(lse2) - got["lse"])) <= 1e-2


def test_fused_rotary_long_positions():
    """Positions up to 40000 (an fp32 angle would be off by 2e-3 rad there): sampled rows."""
    lengths, hq, hkv, d, base = [40000, 300], 2, 1, 128, 10000.0
    cu = wl.cu_seqlens(lengths)
    T = int(cu[-1])
    rng = np.random.Generator(np.random.Philox(key=[63, 7]))
    q, k, v = (round_bf16(rng.standard_normal((T, h, d), dtype=np.float32)) for h in (hq, hkv, hkv))
    scale = 1.0 / float(np.sqrt(d))
    k_rot = round_bf16(ro.rope_packed(k, cu, base=base))
    cu_d = torch.from_numpy(cu).cuda()
    o, lse = binding.varlen_attn_fwd(gu.to_dev(q, "bf16"), gu.to_dev(k_rot, "bf16"), gu.to_dev(v, "bf16"), cu_d, 40000, scale, rope_base=base)
    torch.cuda.synchronize()
    toks = np.array([0, 1, 255, 256, 20000, 39871, 39999, 40000, 40299], dtype=np.int32)
    heads = np.array([0, 1, 0, 1, 0, 1, 0, 1, 0], dtype=np.int32)
    q_rot32 = round_bf16(ro.rope_packed(q, cu, base=base))
    ro_, rl, _ = orc.rows(q_rot32, k_rot, v, None, cu, scale, toks, heads)
    ti, hi = torch.from_numpy(toks.astype(np.int64)).cuda(), torch.from_numpy(heads.astype(np.int64)).cuda()
    gu.check("o[rows]", gu.to_np(o[ti, hi]), ro_, "bf16")
    gu.check("lse[rows]", gu.to_np(lse[hi, ti]), rl, "bf16")
