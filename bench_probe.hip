// Bench-only helper (not part of the product library): sustained-rate probes of the bf16 matrix
// pipe, which bench.py prints beside the roofline to say what this board sustains when the matrix
// pipe is never starved.  The answer depends on the operand DATA (power management lowers the
// clock when operands toggle many bits), so the pattern is an argument.
//   patterns 0 / 1: nothing but v_mfma_f32_32x32x16_bf16 on register operands (zeros / random),
//                   two waves per SIMD, four independent accumulator chains per wave
//   patterns 2 / 3: the same instruction inside the forward kernel's steady-state instruction mix
// Built by __graft_entry__.build() into bench_probe.so; one C entry point, bench_probe_mfma.
#include <hip/hip_runtime.h>

#include "paper_2412_07894_amd/csrc/hyd_device.h"

namespace hyd {

constexpr int kProbeThreads = 512;
constexpr int kProbeMfmaPerIter = 4;

// pattern 0: all operands zero; pattern 1: pseudo-random bf16 values of magnitude around one
__global__ void __launch_bounds__(kProbeThreads) bench_probe_mfma_kernel(float* out, int iters, int pattern) {
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


// The forward kernel's steady-state instruction mix without any of its synchronisation: per MFMA
// one 1 KB operand fragment read from LDS, and per pair of MFMAs two multiply-adds, two
// exponentials, one packed conversion to bf16, one row-sum dot product and one three-way maximum
// (what a 64-key tile costs a wave, divided by its 32 MFMAs).  No barriers, no loads from memory,
// no masks, all waves alike: the rate this loop sustains is what the tile loop could reach if
// everything around the arithmetic were free.  pattern 0 / 1 as above (LDS and register operands).
constexpr int kProbeMixMfmaPerIter = 16;
constexpr int kProbeMixLds = 16384;                    // 16 fragments of 1 KB

__global__ void __launch_bounds__(kProbeThreads, 1) bench_probe_mix_kernel(float* out, int iters, int pattern) {
    __shared__ __attribute__((aligned(16))) char lds[kProbeMixLds];
    uint32_t h = (blockIdx.x * kProbeThreads + threadIdx.x) * 2654435761u + 12345u;
    auto next_pair = [&]() -> uint32_t {
        h = h * 1664525u + 1013904223u;
        const uint32_t lo = 0x3f80u | ((h >> 8) & 0x807fu), hi = 0x3f80u | ((h >> 16) & 0x807fu);
        return pattern ? (lo | (hi << 16)) : 0u;
    };
    for (int i = threadIdx.x; i < kProbeMixLds / 4; i += kProbeThreads) reinterpret_cast<uint32_t*>(lds)[i] = next_pair();
    __syncthreads();
    // fragment f of an iteration sits at byte 1024 * f + 16 * lane: 16 KB, inside the array
    const uint32_t lbase = (uint32_t)(uintptr_t)(lds_char*)lds + (threadIdx.x & 63) * 16;
    bf16x8 qf[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        u32x4 u = {next_pair(), next_pair(), next_pair(), next_pair()};
        qf[k] = as_bf16x8(u);
    }
    f32x16 c[2];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[m][r] = 0.f;
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.01f * i + (threadIdx.x & 7) * 0.1f;
    float lsum = 0.f, mx = 0.f, sc = 0.5f, mr = 1.0f;
    uint32_t pk = 0;
    asm volatile("" : "+v"(sc), "+v"(mr));
    u32x4 kf[4];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(kf[i]) : "v"(lbase), "i"(i * 1024));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kProbeMixMfmaPerIter; ++i) {
            if ((i & 1) == 0) {
                float a = x[i & 7], b = x[(i + 1) & 7];
                asm volatile("v_fma_f32 %0, %0, %1, -%2" : "+v"(a) : "v"(sc), "v"(mr));
                asm volatile("v_fma_f32 %0, %0, %1, -%2" : "+v"(b) : "v"(sc), "v"(mr));
                asm volatile("v_exp_f32 %0, %0" : "+v"(a));
                asm volatile("v_exp_f32 %0, %0" : "+v"(b));
                uint32_t pr;
                asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pr) : "v"(a), "v"(b));
                asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(lsum) : "v"(pr), "v"(0x3f803f80u));
                asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(mx) : "v"(a), "v"(b));
                pk ^= pr;
                x[i & 7] = a * 0.001f + 0.3f;           // keeps the values bounded
                x[(i + 1) & 7] = b;
                asm volatile("" : "+v"(x[i & 7]));
            }
            // LDS reads return in order: fragment i is there once at most the later ones are outstanding
            asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(kf[i & 3]) : "i"(i < 13 ? 3 : 15 - i));
            c[i & 1] = mfma32(as_bf16x8(kf[i & 3]), qf[i >> 1], c[i & 1]);
            if (i + 4 < kProbeMixMfmaPerIter)
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(kf[i & 3]) : "v"(lbase), "i"((i + 4) * 1024));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = lsum + (float)pk + mx;
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[m][r];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += x[i];
    out[blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace hyd

// Runs one probe launch on the null stream, timed with HIP events.  device_out: device,
// float[workgroups * 512].  Returns 0, or 1 (bad argument), 2 (HIP error).
extern "C" int bench_probe_mfma(int workgroups, int iters, int pattern, float* device_out, double* flops, float* ms) {
    using namespace hyd;
    if (!device_out || !flops || !ms || workgroups <= 0 || iters <= 0 || pattern < 0 || pattern > 3) return 1;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 2;
    (void)hipEventRecord(e0, nullptr);
    if (pattern < 2) hipLaunchKernelGGL(bench_probe_mfma_kernel, dim3(workgroups), dim3(kProbeThreads), 0, nullptr, device_out, iters, pattern);
    else hipLaunchKernelGGL(bench_probe_mix_kernel, dim3(workgroups), dim3(kProbeThreads), 0, nullptr, device_out, iters, pattern - 2);
    (void)hipEventRecord(e1, nullptr);
    const bool ok = hipGetLastError() == hipSuccess && hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(ms, e0, e1) == hipSuccess;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *flops = (double)workgroups * (kProbeThreads / 64) * (double)iters * (pattern < 2 ? kProbeMfmaPerIter : kProbeMixMfmaPerIter) *
             (2.0 * 32 * 32 * 16);
    return ok ? 0 : 2;
}
