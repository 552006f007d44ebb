// Sustained-rate probe of the bf16 matrix pipe: nothing but v_mfma_f32_32x32x16_bf16 on register
// operands, two waves per SIMD, four independent accumulator chains per wave.  It answers the
// question the attention kernels' roofline fraction depends on: what this board sustains when the
// matrix pipe is never starved.  The answer depends on the operand DATA (power management lowers
// the clock when operands toggle many bits), so the pattern is an argument.
#pragma once
#include "hyd_device.h"

namespace hyd {

constexpr int kProbeThreads = 512;
constexpr int kProbeMfmaPerIter = 4;

// pattern 0: all operands zero; pattern 1: pseudo-random bf16 values of magnitude around one
__global__ void __launch_bounds__(kProbeThreads) hyd_probe_mfma_kernel(float* out, int iters, int pattern) {
    uint32_t h = (blockIdx.x * kProbeThreads + threadIdx.x) * 2654435761u + 12345u;
    auto next_pair = [&]() -> uint32_t {            // two bf16 values in [1, 2) with random mantissas and signs
        h = h * 1664525u + 1013904223u;
        const uint32_t lo = 0x3f80u | ((h >> 8) & 0x807fu), hi = 0x3f80u | ((h >> 16) & 0x807fu);
        return pattern ? (lo | (hi << 16)) : 0u;
    };
    bf16x8 a[kProbeMfmaPerIter], b[kProbeMfmaPerIter];
#pragma unroll
    for (int m = 0; m < kProbeMfmaPerIter; ++m) {
        u32x4 ua = {next_pair(), next_pair(), next_pair(), next_pair()};
        u32x4 ub = {next_pair(), next_pair(), next_pair(), next_pair()};
        a[m] = as_bf16x8(ua);
        b[m] = as_bf16x8(ub);
    }
    f32x16 c[kProbeMfmaPerIter];
#pragma unroll
    for (int m = 0; m < kProbeMfmaPerIter; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[m][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < kProbeMfmaPerIter; ++m) c[m] = mfma32(a[m], b[m], c[m]);
    }
    float s = 0.f;
#pragma unroll
    for (int m = 0; m < kProbeMfmaPerIter; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[m][r];
    out[blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace hyd
