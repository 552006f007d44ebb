"""The rate probes that bench.py prints beside the roofline (bench-only helper bench_probe.so, not
part of the product library): each pattern runs, reports the floating-point operations it
performed and a positive duration, and its all-zero variants leave zeros behind (a loop of MFMAs on
zero operands, plus, in the mix patterns, bounded softmax-like arithmetic whose result is finite)."""
import ctypes
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("pattern,mfma_per_iter", [(0, 4), (1, 4), (2, 16), (3, 16)])
def test_probe_patterns_run_and_count_their_flops(pattern, mfma_per_iter):
    import torch
    lib = ctypes.CDLL(os.path.join(ROOT, "bench_probe.so"))
    lib.bench_probe_mfma.restype = ctypes.c_int
    lib.bench_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                     ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float)]
    wgs, iters = 64, 50
    out = torch.empty(wgs * 512, dtype=torch.float32, device="cuda")
    flops, ms = ctypes.c_double(0.0), ctypes.c_float(0.0)
    assert lib.bench_probe_mfma(wgs, iters, pattern, out.data_ptr(), ctypes.byref(flops), ctypes.byref(ms)) == 0
    torch.cuda.synchronize()
    assert ms.value > 0.0
    assert flops.value == wgs * 8 * iters * mfma_per_iter * 2.0 * 32 * 32 * 16
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    if pattern == 0:
        assert np.all(got == 0.0)
    assert lib.bench_probe_mfma(wgs, iters, 7, out.data_ptr(), ctypes.byref(flops), ctypes.byref(ms)) == 1
