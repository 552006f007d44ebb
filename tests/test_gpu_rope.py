"""GPU parity of the packed rotary embedding against the fp64 reference.  The kernel's result is
the fp32 rotation rounded once to bf16, so an element may differ from the reference by half a
bf16 step of the result plus fp32 rounding noise, no more."""
import numpy as np
import pytest
import torch

from oracle import rope_oracle as ro
from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def check_rounded(got, ref):
    tol = gu.half_ulp_bf16(ref) * (1 + 1e-3) + 4e-6 * np.maximum(1.0, np.abs(ref))
    err = np.abs(got - ref)
    print(f"rope: max err {err.max():.3e}, max err / tolerance {np.max(err / tol):.3f}, max|ref| {np.abs(ref).max():.3f}", flush=True)
    assert np.all(err <= tol)


@pytest.mark.parametrize("lengths,heads", [([1, 7, 64, 184, 0, 33], 3), ([5000, 300], 2), ([17] * 40, 5)])
def test_rope_forward_inverse_in_place(lengths, heads):
    cu = wl.cu_seqlens(lengths)
    T = int(cu[-1])
    x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.random.default_rng(3).standard_normal((T, heads, 128)).astype(np.float32)))
    xd = gu.to_dev(x, "bf16")
    cu_d = torch.from_numpy(cu).cuda()
    y = binding.rope_packed(xd, cu_d)
    check_rounded(gu.to_np(y), ro.rope_packed(x, cu))
    z = binding.rope_packed(xd, cu_d, inverse=True, base=500000.0)
    check_rounded(gu.to_np(z), ro.rope_packed(x, cu, base=500000.0, inverse=True))
    w = xd.clone()
    binding.rope_packed(w, cu_d, out=w)
    torch.cuda.synchronize()
    assert torch.equal(w, y)                                # in place gives the same bits
    starts = [int(c) for c, L in zip(cu[:-1], lengths) if L > 0]
    assert torch.equal(y[starts], xd[starts])               # every sequence starts at position 0


def test_rope_head_dim_64():
    lengths, heads = [33, 1, 300], 3
    cu = wl.cu_seqlens(lengths)
    T = int(cu[-1])
    x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.random.default_rng(4).standard_normal((T, heads, 64)).astype(np.float32)))
    y = binding.rope_packed(gu.to_dev(x, "bf16"), torch.from_numpy(cu).cuda())
    check_rounded(gu.to_np(y), ro.rope_packed(x, cu))


def test_rope_long_positions_and_rate():
    """One 65536-token sequence (angles up to 65535 rad: fp32 angles would fail here) next to
    short ones, 8 heads; sampled rows against the reference, and the achieved HBM rate."""
    lengths = [65536, 700, 3]
    heads = 8
    cu = wl.cu_seqlens(lengths)
    T = int(cu[-1])
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    xd = torch.randn((T, heads, 128), device="cuda", dtype=torch.float32, generator=g).to(torch.bfloat16)
    cu_d = torch.from_numpy(cu).cuda()
    y = binding.rope_packed(xd, cu_d)
    rows = np.array([0, 1, 2, 4095, 4096, 32767, 65534, 65535, 65536, 65537, 66235, 66236, 66238])
    x_np = gu.to_np(xd[rows])
    sub_cu = np.arange(len(rows) + 1)                       # each sampled row as a sequence of its own...
    pos = ro.positions(cu, T)[rows]
    ref = np.stack([ro.rope_packed(np.concatenate([np.zeros((p, heads, 128)), x_np[i:i + 1]]), [0, p + 1])[p] for i, p in enumerate(pos)])
    check_rounded(gu.to_np(y[rows]), ref)
    binding.enable_kernel_timing(True)
    for _ in range(5):
        binding.rope_packed(xd, cu_d, out=y)
    ms = [t for n, t in binding.kernel_times() if n == "rope_bf16"]
    binding.enable_kernel_timing(False)
    gbs = 2.0 * T * heads * 256 / (min(ms) * 1e-3) / 1e9
    print(f"rope: {T} rows x {heads} heads, {min(ms) * 1e3:.1f} us, {gbs:.0f} GB/s of compulsory traffic (read + write once)", flush=True)
    assert gbs > 1500.0
