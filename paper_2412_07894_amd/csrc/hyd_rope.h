// Rotary position embedding of a packed buffer with the position reset at every sequence start:
// what packing asks of the positional embedding (arXiv 2412.07894, Sec. 2.1: packed sequences must
// keep the positions they would have alone).  Row t of sequence s gets local position
// m = t - cu_seqlens[s]; pair i of a head is (x[i], x[i + d/2]) and turns by m * base^(-2i/d)
// (RoFormer Eq. 34 in its "rotate-half" arrangement); `inverse` turns the other way, which is the
// transpose and carries gradients back.  Angles are formed in double precision: at position 65535
// an fp32 angle is off by up to 4e-3 rad, more than a bf16 result resolves.
// Purely HBM-bound: every element is read once and written once, 16 bytes per lane, whole rows.
#pragma once
#include "hyd_device.h"

namespace hyd {

constexpr int kRopeTok = 16;          // packed rows per workgroup
constexpr int kRopeThreads = 256;

template <int D = kHeadDim>
__global__ void __launch_bounds__(kRopeThreads) hyd_rope_bf16_kernel(const uint16_t* x, const int32_t* __restrict__ cu,
                                                                     int nseq, int T, int heads, double log2_base,
                                                                     int inverse, uint16_t* out) {
    constexpr int kHalf = D / 2;
    __shared__ int pos[kRopeTok];
    __shared__ float cs[kRopeTok][kHalf][2];
    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * kRopeTok;
    if (tid < kRopeTok) {
        const int t = t0 + tid;
        int p = 0;
        if (t < T) {                      // the last sequence that starts at or before row t
            int lo = 0, hi = nseq;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (cu[mid] <= t) lo = mid; else hi = mid - 1;
            }
            p = t - cu[lo];
        }
        pos[tid] = p;
    }
    __syncthreads();
    for (int e = tid; e < kRopeTok * kHalf; e += kRopeThreads) {
        const int r = e / kHalf, i = e % kHalf;
        const double ang = (double)pos[r] * exp2(-(double)(2 * i) / D * log2_base);
        double s, c;
        sincos(inverse ? -ang : ang, &s, &c);
        cs[r][i][0] = (float)c;
        cs[r][i][1] = (float)s;
    }
    __syncthreads();
    // eight lanes per (row, head), D/16 of them at work: lane c owns elements [8c, 8c+8) and their
    // partners [D/2 + 8c, D/2 + 8c + 8)
    const int c8 = tid & 7, slot = tid >> 3;
    const int items = kRopeTok * heads;
    for (int it = slot; it < items; it += kRopeThreads / 8) {
        const int r = it / heads, h = it % heads;
        const int t = t0 + r;
        if (t >= T) break;
        if (D != kHeadDim && c8 >= D / 16) continue;
        const int64_t off = ((int64_t)t * heads + h) * D + 8 * c8;
        const u32x4 lo = *reinterpret_cast<const u32x4*>(x + off);
        const u32x4 hi = *reinterpret_cast<const u32x4*>(x + off + kHalf);
        u32x4 olo, ohi;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float c0 = cs[r][8 * c8 + 2 * e][0], s0 = cs[r][8 * c8 + 2 * e][1];
            const float c1 = cs[r][8 * c8 + 2 * e + 1][0], s1 = cs[r][8 * c8 + 2 * e + 1][1];
            const float a0 = bf16_lo(lo[e]), a1 = bf16_hi(lo[e]), b0 = bf16_lo(hi[e]), b1 = bf16_hi(hi[e]);
            olo[e] = pack_bf16(a0 * c0 - b0 * s0, a1 * c1 - b1 * s1);
            ohi[e] = pack_bf16(b0 * c0 + a0 * s0, b1 * c1 + a1 * s1);
        }
        *reinterpret_cast<u32x4*>(out + off) = olo;
        *reinterpret_cast<u32x4*>(out + off + kHalf) = ohi;
    }
}

}  // namespace hyd
