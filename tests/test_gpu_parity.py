"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle, element by
element on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def full_parity(lengths, hq, hkv, d, dtype, seed, scale=None, host_cu=True):
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, dtype, seed)
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    print(f"\ncase lengths={list(lengths)[:12]}{'...' if len(lengths) > 12 else ''} hq={hq} hkv={hkv} d={d} {dtype} seed={seed} scale={scale}", flush=True)
    got = gu.run_gpu(cu, q, k, v, do, dtype, scale, host_cu=host_cu)
    failures = []
    gu.check_all(got, q, k, v, do, cu, scale, dtype, failures, orc)
    assert not failures, "\n".join(failures)
    return got


def test_config1_fp32():
    cfg = wl.CONFIGS[1]
    lengths = wl.seqlens(1)
    cu = wl.cu_seqlens(lengths)
    T = cfg.total_tokens
    q = wl.normal_tensor(1, "q", T, cfg.hq, cfg.d, "fp32")
    k = wl.normal_tensor(1, "k", T, cfg.hkv, cfg.d, "fp32")
    v = wl.normal_tensor(1, "v", T, cfg.hkv, cfg.d, "fp32")
    do = wl.normal_tensor(1, "do", T, cfg.hq, cfg.d, "fp32")
    print("\nconfig 1", lengths, flush=True)
    got = gu.run_gpu(cu, q, k, v, do, "fp32", cfg.scale)
    o, lse = orc.fwd(q, k, v, cu, cfg.scale)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, cfg.scale)
    for name, ref in (("o", o), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv)):
        gu.check(name, got[name], ref, "fp32")


@pytest.mark.parametrize("lengths,hq,hkv,d", [
    ([1, 7, 64, 184, 65, 0, 130], 4, 2, 64),
    ([200, 3], 3, 1, 128),
])
def test_fp32_small(lengths, hq, hkv, d):
    full_parity(lengths, hq, hkv, d, "fp32", seed=21)


@pytest.mark.parametrize("lengths,hq,hkv", [
    ([1], 1, 1),                                        # a single token
    ([1, 7, 64, 184], 2, 2),                            # config-1 structure in bf16
    ([128, 129, 127, 1, 0, 256, 33], 4, 2),             # tile-boundary lengths, an empty sequence
    ([513, 64, 300], 8, 8),                             # several tiles and ragged tails; 8 heads = partitioned queues
    ([700], 16, 8),                                     # GQA group of 2 with whole groups per queue
    ([90, 1000, 31], 5, 5),                             # head count that stripes items over the queues
])
def test_bf16_small(lengths, hq, hkv):
    full_parity(lengths, hq, hkv, 128, "bf16", seed=31)


@pytest.mark.parametrize("lengths,hq,hkv", [
    ([1, 7, 64, 184], 2, 2),
    ([128, 129, 127, 1, 0, 256, 33], 4, 2),
    ([513, 64, 300], 8, 8),
    ([90, 1000, 31], 6, 3),
    ([2100], 4, 1),
])
def test_bf16_head_dim_64(lengths, hq, hkv):
    """The bf16 kernels at head_dim 64: same tiles, half the contraction steps and output blocks."""
    full_parity(lengths, hq, hkv, 64, "bf16", seed=37)


def test_bf16_head_dim_64_no_cross_contamination():
    # rows of 128 bytes sit next to each other in memory (head h+1 follows head h): the loads that
    # cover only half of a 256-byte LDS row must not pick up the neighbour
    lengths, hq, hkv, d = [300, 129, 200], 4, 2, 64
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 38)
    scale = 1.0 / np.sqrt(d)
    a = gu.run_gpu(cu, q, k, v, do, "bf16", scale)
    q2, k2, v2, do2 = q.copy(), k.copy(), v.copy(), do.copy()
    q2[:, 1] *= 3; k2[:, 1] *= -2; v2[:, 1] += 1; do2[:, 1] *= 0.5          # heads 1 (query) and 1 (KV) change
    b = gu.run_gpu(cu, q2, k2, v2, do2, "bf16", scale)
    # query heads 0, 1 use KV head 0; heads 2, 3 use KV head 1: head 0 and KV head 0's share from head 0 stay
    assert np.array_equal(a["o"][:, 0], b["o"][:, 0]) and np.array_equal(a["lse"][0], b["lse"][0])
    assert np.array_equal(a["dq"][:, 0], b["dq"][:, 0])
    assert not np.array_equal(a["o"][:, 2], b["o"][:, 2])


def test_bf16_many_heads():
    # 160 query heads: the statistics pass of the backward takes fewer tokens per workgroup
    full_parity([70, 33, 130], 160, 40, 64, "bf16", seed=39)


def test_bf16_thousands_of_short_sequences():
    # more sequences than the schedule prelude has threads, every item a single partial tile,
    # empty sequences in between
    rng = np.random.default_rng(5)
    lengths = [int(x) for x in rng.integers(0, 41, size=3000)]
    full_parity(lengths, 8, 2, 128, "bf16", seed=41)


def test_bf16_one_long_sequence_among_tiny_ones():
    # levels 1..24 from one sequence only, next to many one-tile sequences: long ramp in the item
    # list, queues that run dry at different times (work stealing)
    lengths = [3, 6100, 1, 17, 64, 2, 255, 9]
    full_parity(lengths, 6, 3, 128, "bf16", seed=43)


def test_bf16_without_host_seqlens_and_other_scale():
    full_parity([300, 45, 128], 4, 1, 128, "bf16", seed=32, scale=0.05, host_cu=False)


def test_bf16_scale_zero_is_uniform_attention():
    got = full_parity([70, 200], 2, 2, 128, "bf16", seed=33, scale=0.0)
    assert np.allclose(got["lse"][:, 69], np.log(70.0), atol=1e-5)


def test_bf16_negative_scale():
    full_parity([150, 260], 2, 1, 128, "bf16", seed=34, scale=-0.07)


def test_backward_alone_with_oracle_forward():
    """Isolates the backward: it is fed the oracle's O (rounded to bf16) and LSE."""
    lengths, hq, hkv, d = [257, 100], 4, 2, 128
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 35)
    scale = 1.0 / np.sqrt(d)
    o, lse = orc.fwd(q, k, v, cu, scale)
    o_b = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(o.astype(np.float32)))
    got = gu.run_gpu(cu, q, k, v, do, "bf16", scale, o_lse=(o_b, lse))
    # the reference is the oracle's backward of exactly what the GPU backward was handed
    dq, dk, dv = orc.bwd_given(q, k, v, do, o_b, lse.astype(np.float32), cu, scale)
    for name, ref in (("dq", dq), ("dk", dk), ("dv", dv)):
        gu.check(name, got[name], ref, "bf16")


def test_bitwise_reproducible_and_no_cross_contamination():
    lengths, hq, hkv, d = [300, 129, 700], 8, 2, 128
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 36)
    scale = 1.0 / np.sqrt(d)
    a = gu.run_gpu(cu, q, k, v, do, "bf16", scale)
    b = gu.run_gpu(cu, q, k, v, do, "bf16", scale)
    for name in a:
        assert np.array_equal(a[name], b[name]), name
    # perturb the middle sequence: the others must not change by a single bit
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[cu[1]:cu[2]] *= 2; k2[cu[1]:cu[2]] *= -1; v2[cu[1]:cu[2]] *= 0.5
    c = gu.run_gpu(cu, q2, k2, v2, do, "bf16", scale)
    keep = np.r_[0:cu[1], cu[2]:cu[3]]
    for name in ("o", "dq", "dk", "dv"):
        assert np.array_equal(a[name][keep], c[name][keep]), name
    assert np.array_equal(a["lse"][:, keep], c["lse"][:, keep])


def test_outputs_do_not_spill_past_their_rows():
    """Canary rows around every output must survive."""
    lengths, hq, hkv, d = [130, 61], 2, 1, 128
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 37)
    T = int(cu[-1])
    scale = 1.0 / np.sqrt(d)
    pad = 64
    cu_d = torch.from_numpy(cu).cuda()
    qd, kd, vd, dod = (gu.to_dev(x, "bf16") for x in (q, k, v, do))
    def guarded(rows, heads):
        buf = torch.full((rows + 2 * pad, heads, d), 7.0, dtype=torch.bfloat16, device="cuda")
        return buf, buf[pad:pad + rows]
    ob, o = guarded(T, hq); dqb, dq = guarded(T, hq); dkb, dk = guarded(T, hkv); dvb, dv = guarded(T, hkv)
    lseb = torch.full((hq * T + 2 * pad,), 7.0, dtype=torch.float32, device="cuda")
    lse = lseb[pad:pad + hq * T].view(hq, T)
    binding.varlen_attn_fwd(qd, kd, vd, cu_d, 130, scale, out=o, lse=lse)
    binding.varlen_attn_bwd(qd, kd, vd, o, lse, dod, cu_d, 130, scale, dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    for buf, rows in ((ob, T), (dqb, T), (dkb, T), (dvb, T)):
        assert torch.all(buf[:pad] == 7.0) and torch.all(buf[pad + rows:] == 7.0)
    assert torch.all(lseb[:pad] == 7.0) and torch.all(lseb[pad + hq * T:] == 7.0)


def test_empty_inputs_are_noops():
    z = torch.empty((0, 2, 128), dtype=torch.bfloat16, device="cuda")
    cu0 = torch.zeros(1, dtype=torch.int32, device="cuda")
    o, lse = binding.varlen_attn_fwd(z, z, z, cu0, 0, 0.1)
    assert o.shape == (0, 2, 128) and lse.shape == (2, 0)
    binding.varlen_attn_bwd(z, z, z, o, lse, z, cu0, 0, 0.1)
    torch.cuda.synchronize()
