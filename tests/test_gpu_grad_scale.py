"""The backward's handling of the scale of dO.  Its products run in fp16, whose exponent range is
narrow, so dO is scaled into range by powers of two (one per tensor for dK and dV, one per row for
dQ) that are undone in the results.  Scaling by a power of two is exact, so the results must
follow the scale of dO bit for bit: gradients of a loss divided by a million are the gradients
divided by a million."""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def grads(cu, q, k, v, do, scale):
    cu_d = torch.from_numpy(cu).cuda()
    qd, kd, vd, dod = (gu.to_dev(x, "bf16") for x in (q, k, v, do))
    ml = int(np.diff(cu).max())
    o, lse = binding.varlen_attn_fwd(qd, kd, vd, cu_d, ml, scale)
    dq, dk, dv = binding.varlen_attn_bwd(qd, kd, vd, o, lse, dod, cu_d, ml, scale)
    torch.cuda.synchronize()
    return dq.float(), dk.float(), dv.float()


@pytest.mark.parametrize("log2_gain", [-20, -40, 12])
def test_gradients_follow_a_power_of_two_scale_of_do_bit_for_bit(log2_gain):
    lengths, hq, hkv, d = [300, 129, 700, 1], 4, 2, 128
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 81)
    scale = 1.0 / float(np.sqrt(d))
    gain = np.float32(2.0 ** log2_gain)
    base = grads(cu, q, k, v, do, scale)
    scaled = grads(cu, q, k, v, do * gain, scale)
    print(f"\ndO x 2^{log2_gain}: max |dq| {float(scaled[0].abs().max()):.3e}", flush=True)
    for name, a, b in zip(("dq", "dk", "dv"), base, scaled):
        assert torch.equal(a * float(gain), b), name


def test_rows_with_very_different_gradient_scales():
    """Every (token, head) row of dO gets its own power of two between 2^-14 and 1, some rows are
    zero.  dQ is row-wise and scaled per row: each row must equal the unscaled run's row times
    its factor, bit for bit.  dK and dV sum over rows and are compared with the oracle."""
    lengths, hq, hkv, d = [513, 64, 300], 4, 2, 128
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 82)
    scale = 1.0 / float(np.sqrt(d))
    rng = np.random.default_rng(9)
    T = int(cu[-1])
    f = (2.0 ** rng.integers(-14, 1, size=(T, hq))).astype(np.float32)
    f[rng.random((T, hq)) < 0.05] = 0.0
    do2 = do * f[:, :, None]
    base = grads(cu, q, k, v, do, scale)
    got = grads(cu, q, k, v, do2, scale)
    assert torch.equal(base[0] * torch.from_numpy(f).cuda()[:, :, None], got[0])
    _, rdk, rdv = orc.bwd(q, k, v, do2, cu, scale)
    gu.check("dk", got[1].cpu().numpy().astype(np.float64), rdk, "bf16")
    gu.check("dv", got[2].cpu().numpy().astype(np.float64), rdv, "bf16")
    # relative to the size of these gradients the bar above is loose: rel-L2 is the tight one here
