"""GPU parity on seeded random shapes: sequence counts, lengths that straddle every tile size in
use (32-row blocks, 64-key tiles, 128-key and 256-row work items), head counts and group sizes
drawn at random; the plain calls and, for sequences long enough, one range visit.  Each case is
small enough for the full fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from oracle import range_oracle as rorc
from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    nseq = int(rng.integers(1, 9))
    edges = np.array([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 255, 256, 257, 320, 511, 513, 700])
    lengths = [int(rng.choice(edges)) if rng.random() < 0.7 else int(rng.integers(0, 900)) for _ in range(nseq)]
    if sum(lengths) == 0:
        lengths[0] = 5
    hkv = int(rng.choice([1, 2, 3, 8]))
    g = int(rng.choice([1, 2, 4]))
    rng.choice([0, 1, 2])           # (a draw that older versions of this file spent on the scale)
    return lengths, hkv * g, hkv


@pytest.mark.parametrize("seed", range(10))
def test_random_shape(seed):
    lengths, hq, hkv = draw(seed)
    d = 64 if seed in (1, 4, 7) else 128
    scale = 1.0 / float(np.sqrt(d))         # the benchmark configurations' scale, unit-variance dO
    print(f"\nrandom shape seed={seed} lengths={lengths} hq={hq} hkv={hkv} d={d} scale={scale:.4f}", flush=True)
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 70 + seed)
    got = gu.run_gpu(cu, q, k, v, do, "bf16", scale, host_cu=bool(seed & 1))
    failures = []
    gu.check_all(got, q, k, v, do, cu, scale, "bf16", failures, orc)
    assert not failures, "\n".join(failures)
    # one range visit: queries from row 256 on against the keys before them
    if max(lengths) > 256:
        A = binding.RANGE_ALIGN
        ranges = [(A, 4 * A, 0, A)] * len(lengths)
        T = int(cu[-1])
        dev = [gu.to_dev(x, "bf16") for x in (q, k, v)]
        cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
        out = torch.full((T, hq, d), 3.0, dtype=torch.bfloat16, device="cuda")
        ls = torch.full((hq, T), 9.0, dtype=torch.float32, device="cuda")
        binding.varlen_attn_fwd_range(dev[0], dev[1], dev[2], cu_d, ranges, max(lengths), scale, out, ls,
                                      cu_seqlens_host=[int(x) for x in cu])
        torch.cuda.synchronize()
        o_ref, l_ref = rorc.fwd_range(q, k, v, cu, scale, [(r[0], r[1]) for r in ranges], [(r[2], r[3]) for r in ranges])
        inq = ~np.isnan(l_ref[0])
        assert inq.any()
        gu.check("o[visit]", gu.to_np(out)[inq], o_ref[inq], "bf16")
        gu.check("lse[visit]", gu.to_np(ls)[:, inq], l_ref[:, inq], "bf16")
        assert np.all(gu.to_np(out)[~inq] == 3.0) and np.all(gu.to_np(ls)[:, ~inq] == 9.0)
