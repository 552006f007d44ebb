// Rotary position embedding applied to rows that sit in registers: the Q rows of a work item when
// the forward and the dQ kernel pick them up, and the dQ rows before they are written (inverse
// rotation, i.e. the transpose, which carries the gradient back to the unrotated Q).  Packing
// asks for positions that restart in every packed sequence (arXiv 2412.07894, Sec. 2.1); a work
// item knows the LOCAL position of each of its rows, so the reset costs nothing here, and Q needs
// no pass of its own through HBM (K, which every query tile of a sequence streams again, is
// rotated once per layer by hyd_rope_packed).  Pairing and angles as in hyd_rope.h: pair i of a
// head is (x[i], x[i + d/2]) and turns by pos * base^(-2i/d).
//
// Angles: the table holds base^(-2i/d) / (2 pi) in double precision; pos * table[i] is formed in
// double, reduced to [0, 1) revolutions there (at position 65535 an fp32 angle would be off by
// 4e-3 rad) and handed to v_sin_f32 / v_cos_f32, which take revolutions.
#pragma once
#include "hyd_device.h"

namespace hyd {

constexpr double kInvTwoPi = 0.15915494309189533576888;

// Writes the table: pairs i = tid .. half_d-1 (any number of threads may call it).
__device__ __forceinline__ void rope_table_fill(double* tab, int half_d, double log2_base, int tid, int nthreads) {
    for (int i = tid; i < half_d; i += nthreads) tab[i] = exp2(-(double)i / (double)half_d * log2_base) * kInvTwoPi;
}

// cos and sin of the N consecutive pairs i0 .. i0+N-1 at position `pos`; `inverse` negates the angle.
template <int N>
__device__ __forceinline__ void rope_cos_sin(const double* __restrict__ tab, int i0, int pos, bool inverse, float (&c)[N], float (&s)[N]) {
    const double p = (double)pos;
#pragma unroll
    for (int e = 0; e < N; ++e) {
        const double rev = p * tab[i0 + e];
        const float r = (float)(rev - __builtin_floor(rev));
        c[e] = __builtin_amdgcn_cosf(r);
        const float sv = __builtin_amdgcn_sinf(r);
        s[e] = inverse ? -sv : sv;
    }
}

// Row fragments x[ks] (lane: one row; fragment ks holds elements 16 ks + 8 half + {0..7} as four
// packed bf16 pairs): rotated in place and rounded to bf16, which is what a rotary pass of its
// own would have left in HBM - the forward and the backward must see the SAME rotated Q, or the
// backward's P = exp(s - LSE) no longer matches the LSE the forward stored.  F16: the bf16 values
// are then repacked as fp16 (exact) for the fp16 matrix products of the backward.
template <int D, bool F16>
__device__ __forceinline__ void rope_row_frags(u32x4 (&x)[D / 16], const double* __restrict__ tab, int pos, int half) {
    constexpr int NP = D / 32;                      // fragments per half of the head dimension
#pragma unroll
    for (int a = 0; a < NP; ++a) {
        float c[8], s[8];
        rope_cos_sin<8>(tab, 16 * a + 8 * half, pos, false, c, s);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lo = x[a][e], hi = x[a + NP][e];
            const float a0 = bf16_lo(lo), a1 = bf16_hi(lo), b0 = bf16_lo(hi), b1 = bf16_hi(hi);
            const float y0 = a0 * c[2 * e] - b0 * s[2 * e], y1 = a1 * c[2 * e + 1] - b1 * s[2 * e + 1];
            const float z0 = b0 * c[2 * e] + a0 * s[2 * e], z1 = b1 * c[2 * e + 1] + a1 * s[2 * e + 1];
            const uint32_t yb = pack_bf16(y0, y1), zb = pack_bf16(z0, z1);
            x[a][e] = F16 ? bf16x2_to_f16x2(yb) : yb;
            x[a + NP][e] = F16 ? bf16x2_to_f16x2(zb) : zb;
        }
    }
}

// Transposed accumulators acc[db][r] (lane: one row; element 32 db + 8 (r / 4) + 4 half + r % 4
// of it): inverse rotation in place.
template <int D>
__device__ __forceinline__ void rope_acc_inverse(f32x16 (&acc)[D / 32], const double* __restrict__ tab, int pos, int half) {
    constexpr int NP = D / 64;
#pragma unroll
    for (int db = 0; db < NP; ++db) {
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            float c[4], s[4];
            rope_cos_sin<4>(tab, 32 * db + 8 * rq + 4 * half, pos, true, c, s);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const float g1 = acc[db][4 * rq + m], g2 = acc[db + NP][4 * rq + m];
                acc[db][4 * rq + m] = g1 * c[m] - g2 * s[m];
                acc[db + NP][4 * rq + m] = g2 * c[m] + g1 * s[m];
            }
        }
    }
}

}  // namespace hyd
