// Merge of two partial attention results over the same rows (context parallelism: each partial
// comes from one chunk of the keys, arXiv 2412.07894 Sec. 2.1).  With LSE_x = ln sum exp(s) over
// the keys of partial x, the softmax over the union of the keys is
//     LSE = ln(exp(LSE_a) + exp(LSE_b)),   O = exp(LSE_a - LSE) O_a + exp(LSE_b - LSE) O_b;
// a partial that saw no key carries LSE = -inf and O = 0 and is the neutral element.
// Purely HBM-bound: 16 lanes per row, 16 bytes per lane, every byte read and written once.
#pragma once
#include "hyd_device.h"

namespace hyd {

// o_out / lse_out may alias either input (each lane reads what it overwrites before writing it).
template <int D = kHeadDim>
__global__ void __launch_bounds__(256) hyd_merge_bf16_kernel(const uint16_t* o_a, const float* lse_a,
                                                            const uint16_t* o_b, const float* lse_b,
                                                            uint16_t* o_out, float* lse_out, int T, int hq) {
    const int64_t n_rows = (int64_t)T * hq;
    const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int c = threadIdx.x & 15;
    if (row >= n_rows || (D != kHeadDim && c >= D / 8)) return;
    const int t = (int)(row / hq), h = (int)(row % hq);
    const int64_t si = (int64_t)h * T + t;
    const float la = lse_a[si], lb = lse_b[si];
    const float m = fmaxf(la, lb);
    float ca = 0.f, cb = 0.f, lse = -INFINITY;
    if (m > -INFINITY) {
        constexpr float kL2e = 1.44269504088896340736f, kLn2 = 0.69314718055994530942f;
        const float wa = __builtin_amdgcn_exp2f((la - m) * kL2e), wb = __builtin_amdgcn_exp2f((lb - m) * kL2e);
        const float tot = wa + wb;                        // in [1, 2]
        lse = m + __builtin_amdgcn_logf(tot) * kLn2;
        const float inv = 1.f / tot;
        ca = wa * inv; cb = wb * inv;
    }
    const u32x4 a = *reinterpret_cast<const u32x4*>(o_a + row * D + c * 8);
    const u32x4 b = *reinterpret_cast<const u32x4*>(o_b + row * D + c * 8);
    u32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        // a weight of zero must also silence a partial whose unwritten rows hold non-finite bits
        const float lo = (ca != 0.f ? ca * bf16_lo(a[e]) : 0.f) + (cb != 0.f ? cb * bf16_lo(b[e]) : 0.f);
        const float hi = (ca != 0.f ? ca * bf16_hi(a[e]) : 0.f) + (cb != 0.f ? cb * bf16_hi(b[e]) : 0.f);
        r[e] = pack_bf16(lo, hi);
    }
    *reinterpret_cast<u32x4*>(o_out + row * D + c * 8) = r;
    if (c == 0) lse_out[si] = lse;
}

}  // namespace hyd
