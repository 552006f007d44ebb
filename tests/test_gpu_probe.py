"""The rate probes that bench.py prints beside the roofline: each pattern runs, reports the
floating-point operations it performed, and its all-zero variants leave zeros behind (a loop of
MFMAs on zero operands, plus — in the mix patterns — bounded softmax-like arithmetic whose result
is finite)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pattern,mfma_per_iter", [(0, 4), (1, 4), (2, 16), (3, 16)])
def test_probe_patterns_run_and_count_their_flops(pattern, mfma_per_iter):
    import torch
    from paper_2412_07894_amd import binding
    wgs, iters = 64, 50
    binding.enable_kernel_timing(True)
    try:
        flops, out = binding.probe_mfma(wgs, iters, pattern)
        (name, ms), = binding.kernel_times()
    finally:
        binding.enable_kernel_timing(False)
    torch.cuda.synchronize()
    assert name == "probe_mfma" and ms > 0.0
    assert flops == wgs * 8 * iters * mfma_per_iter * 2.0 * 32 * 32 * 16
    got = out.cpu().numpy()
    assert got.shape == (wgs * 512,) and np.all(np.isfinite(got))
    if pattern == 0:
        assert np.all(got == 0.0)
