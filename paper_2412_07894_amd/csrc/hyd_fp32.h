// fp32 kernels: the same operation in plain fp32 FMA arithmetic, one thread per query row (forward,
// dQ) or per key row (dK/dV).  This path exists for fp32 inputs (tolerance 1e-5) and has no
// throughput target; it shares the work-item schedule (tile = 64 rows) with the bf16 path.
// K/V (or Q/dO) rows are read with wave-uniform addresses straight from global memory.
#pragma once
#include "hyd_sched.h"

namespace hyd {

constexpr int kF32Tile = 64;
template <int D> constexpr int f32_dkdv_lds() { return 2 * D * kF32Tile * 4 + 64; }

struct F32Params {
    const float* q; const float* k; const float* v; const float* o; const float* d_o;
    const float* lse_in; const float* D;
    float* o_out; float* lse_out; float* D_out;
    float* dq; float* dk; float* dv;
    int T, hq, hkv;
    float scale;
    const int* hdr; int* cursors; const int* items;
    HeadMap hm;
    WgTrace tr;
};

template <int D>
__device__ __forceinline__ float dot_row(const float (&a)[D], const float* __restrict__ b) {
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < D; ++c) acc = __builtin_fmaf(a[c], b[c], acc);
    return acc;
}

template <int D>
__global__ void __launch_bounds__(kF32Tile) hyd_fwd_fp32_kernel(F32Params p) {
    __shared__ int slot[kSlotInts];
    const int tid = threadIdx.x;
    const int G = p.hq / p.hkv;
    WorkFetcher wf;
    WorkItem wi;
    for (bool have = wf.first(p.hm, p.hdr, p.cursors, p.items, slot, wi); have; have = wf.next(p.hm, p.cursors, p.items, slot, wi)) {
        const int lev = wi.lev, head = wi.head, row0 = wi.row0, L = wi.len;
        const int q0 = (lev - 1) * kF32Tile;
        const int i = q0 + tid;
        const bool valid = i < L;
        const int kend = min(L, q0 + kF32Tile);
        const int g = head / G;
        float q[D], o[D];
        const float* qp = p.q + ((int64_t)(row0 + (valid ? i : 0)) * p.hq + head) * D;
#pragma unroll
        for (int c = 0; c < D; ++c) { q[c] = qp[c]; o[c] = 0.f; }
        float m = -INFINITY, l = 0.f;
        for (int j = 0; j < kend; ++j) {
            const float* kp = p.k + ((int64_t)(row0 + j) * p.hkv + g) * D;
            const float* vp = p.v + ((int64_t)(row0 + j) * p.hkv + g) * D;
            if (valid && j <= i) {
                const float s = p.scale * dot_row<D>(q, kp);
                if (s > m) {
                    const float alpha = expf(m - s);
                    l *= alpha;
#pragma unroll
                    for (int c = 0; c < D; ++c) o[c] *= alpha;
                    m = s;
                }
                const float pr = expf(s - m);
                l += pr;
#pragma unroll
                for (int c = 0; c < D; ++c) o[c] = __builtin_fmaf(pr, vp[c], o[c]);
            }
        }
        if (valid) {
            const float inv = 1.f / l;
            float* op = p.o_out + ((int64_t)(row0 + i) * p.hq + head) * D;
#pragma unroll
            for (int c = 0; c < D; ++c) op[c] = o[c] * inv;
            p.lse_out[(int64_t)head * p.T + row0 + i] = m + logf(l);
        }
    }
}

template <int D>
__global__ void __launch_bounds__(256) hyd_bwd_rowdot_fp32_kernel(const float* __restrict__ o,
                                                                 const float* __restrict__ d_o,
                                                                 float* __restrict__ Dv, int T, int hq) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= (int64_t)T * hq) return;
    float acc = 0.f;
    for (int c = 0; c < D; ++c) acc = __builtin_fmaf(o[row * D + c], d_o[row * D + c], acc);
    Dv[(row % hq) * T + row / hq] = acc;
}

template <int D>
__global__ void __launch_bounds__(kF32Tile) hyd_bwd_dq_fp32_kernel(F32Params p) {
    __shared__ int slot[kSlotInts];
    const int tid = threadIdx.x;
    const int G = p.hq / p.hkv;
    WorkFetcher wf;
    WorkItem wi;
    for (bool have = wf.first(p.hm, p.hdr, p.cursors, p.items, slot, wi); have; have = wf.next(p.hm, p.cursors, p.items, slot, wi)) {
        const int lev = wi.lev, head = wi.head, row0 = wi.row0, L = wi.len;
        const int q0 = (lev - 1) * kF32Tile;
        const int i = q0 + tid;
        const bool valid = i < L;
        const int kend = min(L, q0 + kF32Tile);
        const int g = head / G;
        float q[D], g_o[D], dq[D];
        const int64_t qoff = ((int64_t)(row0 + (valid ? i : 0)) * p.hq + head) * D;
#pragma unroll
        for (int c = 0; c < D; ++c) { q[c] = p.q[qoff + c]; g_o[c] = p.d_o[qoff + c]; dq[c] = 0.f; }
        const int64_t at = (int64_t)head * p.T + row0 + (valid ? i : 0);
        const float lse = p.lse_in[at], Di = p.D[at];
        for (int j = 0; j < kend; ++j) {
            const float* kp = p.k + ((int64_t)(row0 + j) * p.hkv + g) * D;
            const float* vp = p.v + ((int64_t)(row0 + j) * p.hkv + g) * D;
            if (valid && j <= i) {
                const float pr = expf(p.scale * dot_row<D>(q, kp) - lse);
                const float ds = pr * (dot_row<D>(g_o, vp) - Di);
#pragma unroll
                for (int c = 0; c < D; ++c) dq[c] = __builtin_fmaf(ds, kp[c], dq[c]);
            }
        }
        if (valid) {
#pragma unroll
            for (int c = 0; c < D; ++c) p.dq[qoff + c] = dq[c] * p.scale;
        }
    }
}

template <int D>
__global__ void __launch_bounds__(kF32Tile) hyd_bwd_dkdv_fp32_kernel(F32Params p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float* acc_k = reinterpret_cast<float*>(smem);                  // [c][thread]
    float* acc_v = acc_k + D * kF32Tile;
    int* slot = reinterpret_cast<int*>(acc_v + D * kF32Tile);
    const int tid = threadIdx.x;
    const int G = p.hq / p.hkv;
    WorkFetcher wf;
    WorkItem wi;
    for (bool have = wf.first(p.hm, p.hdr, p.cursors, p.items, slot, wi); have; have = wf.next(p.hm, p.cursors, p.items, slot, wi)) {
        const int lev = wi.lev, g = wi.head, row0 = wi.row0, L = wi.len;
        const int n_tiles = (L + kF32Tile - 1) / kF32Tile;
        const int j0 = (n_tiles - lev) * kF32Tile;
        const int j = j0 + tid;
        const bool valid = j < L;
        float kr[D], vr[D];
        const int64_t koff = ((int64_t)(row0 + (valid ? j : 0)) * p.hkv + g) * D;
#pragma unroll
        for (int c = 0; c < D; ++c) {
            kr[c] = p.k[koff + c]; vr[c] = p.v[koff + c];
            acc_k[c * kF32Tile + tid] = 0.f; acc_v[c * kF32Tile + tid] = 0.f;
        }
        for (int h = g * G; h < (g + 1) * G; ++h) {
            for (int i = j0; i < L; ++i) {
                const float* qp = p.q + ((int64_t)(row0 + i) * p.hq + h) * D;
                const float* gp = p.d_o + ((int64_t)(row0 + i) * p.hq + h) * D;
                const float lse = p.lse_in[(int64_t)h * p.T + row0 + i];
                const float Di = p.D[(int64_t)h * p.T + row0 + i];
                if (valid && i >= j) {
                    const float pr = expf(p.scale * dot_row<D>(kr, qp) - lse);
                    const float ds = pr * (dot_row<D>(vr, gp) - Di);
#pragma unroll
                    for (int c = 0; c < D; ++c) {
                        acc_v[c * kF32Tile + tid] = __builtin_fmaf(pr, gp[c], acc_v[c * kF32Tile + tid]);
                        acc_k[c * kF32Tile + tid] = __builtin_fmaf(ds, qp[c], acc_k[c * kF32Tile + tid]);
                    }
                }
            }
        }
        if (valid) {
#pragma unroll
            for (int c = 0; c < D; ++c) {
                p.dk[koff + c] = acc_k[c * kF32Tile + tid] * p.scale;
                p.dv[koff + c] = acc_v[c * kF32Tile + tid];
            }
        }
    }
}

}  // namespace hyd
