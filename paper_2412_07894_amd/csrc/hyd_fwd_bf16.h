// bf16 forward kernel: block-diagonal causal flash-style tile loop on MFMA with fp32 accumulation.
//
// Work item = (sequence, 128-row query tile, query head).  A workgroup has 4 waves; wave w owns
// query rows 32w..32w+31 of the tile for the whole item, so the online softmax never crosses
// waves.  K and V tiles of 64 keys are staged through LDS (double buffered, one barrier per tile)
// and shared by the 4 waves.
//
// Orientation.  Scores are computed transposed, S^T[key][q] = K Q^T, so that in the accumulator
// lane map (see mfma32) a lane owns ONE query row (column l%32) and 16 keys per 32-key block:
// the row maximum and row sum are in-lane reductions plus one exchange with the other half of
// the wave, and the softmax statistics m, l and the rescale factor are per-lane scalars.  The
// probabilities then feed the second product O^T[d][q] = V^T P^T directly as the B operand
// (contraction index = key = accumulator row), while V^T fragments come out of the row-major V
// tile with the transposing LDS read.
#pragma once
#include <type_traits>

#include "hyd_sched.h"

namespace hyd {

constexpr int kFwdBM = 128, kFwdBN = 64, kFwdThreads = 256;
constexpr int kFwdTileBytes = kFwdBN * kRowBytes;                 // 16 KB
constexpr int kFwdLds = 4 * kFwdTileBytes + 64;                   // K,V x 2 buffers + work slot

struct FwdParams {
    const uint16_t* q; const uint16_t* k; const uint16_t* v;
    uint16_t* o; float* lse;
    const int32_t* cu;
    int T, hq, hkv;
    float scale_log2;                 // softmax_scale * log2(e)
    const int* hdr; int* cursors; const int* items;
    HeadMap hm;
    WgTrace tr;
};

template <bool MASK>
__device__ __forceinline__ void fwd_tile(const char* Kt, const char* Vt, const FragAddr& fa,
                                         const bf16x8 (&qf)[8], f32x16 (&acc_o)[4], float& m_run,
                                         float& l_run, float scale_log2, int key0, int qrow, int half) {
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
#ifdef HYD_ABL_NOLDS_K
        for (int kb = 0; kb < 2; ++kb) s[kb] = mfma32(frag_row(Kt, fa, kb, 0), qf[ks], s[kb]);
#else
        for (int kb = 0; kb < 2; ++kb) s[kb] = mfma32(frag_row(Kt, fa, kb, ks), qf[ks], s[kb]);
#endif
    }
#ifdef HYD_ABL_NOSOFTMAX
    uint32_t pk[2][8];
    for (int kb = 0; kb < 2; ++kb) for (int r = 0; r < 16; r += 2) pk[kb][r >> 1] = pack_bf16(s[kb][r], s[kb][r + 1]);
    l_run += 1.f; m_run = 0.f;
#else
    // row maximum of the raw scores over visible keys (scale_log2 >= 0 here: a negative softmax
    // scale has been folded into the sign of the Q fragments)
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float x = s[kb][r];
            if (MASK) {
                const int key = key0 + 32 * kb + 8 * (r >> 2) + 4 * half + (r & 3);
                if (key > qrow) x = -INFINITY;
            }
            mx = fmaxf(mx, x);
        }
    }
    mx = fmaxf(mx, shfl_xor32(mx));
    const float m_new = fmaxf(m_run, mx * scale_log2);
    if (__any(m_new > m_run)) {         // rescale only when some row's maximum moved
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[db][r] *= alpha;
        m_run = m_new;
    }
    uint32_t pk[2][8];
    float lsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            float t0 = __builtin_fmaf(s[kb][r], scale_log2, -m_run);
            float t1 = __builtin_fmaf(s[kb][r + 1], scale_log2, -m_run);
            if (MASK) {
                const int key = key0 + 32 * kb + 8 * (r >> 2) + 4 * half + (r & 3);
                if (key > qrow) t0 = -INFINITY;
                if (key + 1 > qrow) t1 = -INFINITY;
            }
            const float p0 = __builtin_amdgcn_exp2f(t0), p1 = __builtin_amdgcn_exp2f(t1);
            lsum += p0 + p1;
            pk[kb][r >> 1] = pack_bf16(p0, p1);
        }
    }
    l_run += lsum;
#endif
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        u32x4 pv = {pk[b >> 1][4 * (b & 1) + 0], pk[b >> 1][4 * (b & 1) + 1],
                    pk[b >> 1][4 * (b & 1) + 2], pk[b >> 1][4 * (b & 1) + 3]};
        const bf16x8 pb = as_bf16x8(pv);
#ifdef HYD_ABL_NOLDS_V
        const bf16x8 va = frag_col(Vt, fa, b, 0);
        for (int db = 0; db < 4; ++db) acc_o[db] = mfma32(va, pb, acc_o[db]);
#else
#pragma unroll
        for (int db = 0; db < 4; ++db) acc_o[db] = mfma32(frag_col(Vt, fa, b, db), pb, acc_o[db]);
#endif
    }
}

__global__ void __launch_bounds__(kFwdThreads, 2) hyd_fwd_bf16_kernel(FwdParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int* slot = reinterpret_cast<int*>(smem + 4 * kFwdTileBytes);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int G = p.hq / p.hkv;
    const int64_t q_stride = (int64_t)p.hq * kHeadDim, kv_stride = (int64_t)p.hkv * kHeadDim;
    const unsigned long long t_start = p.tr.rec ? wall_clock64() : 0ull;
    unsigned long long n_done = 0;

    FragAddr fa;
    fa.init(lane);
    TileMover<kFwdBN, kFwdThreads> mk, mv;
    mk.init(tid, (uint32_t)kv_stride * 2);
    mv.init(tid, (uint32_t)kv_stride * 2);
    const uint32_t tile_bytes = kFwdBN * (uint32_t)kv_stride * 2;     // one K/V tile in global memory
    // scale * s = |scale| * (-s): a negative scale flips the sign bits of the Q fragments instead
    const float scale_log2 = fabsf(p.scale_log2);
    const uint32_t sign_flip = p.scale_log2 < 0.f ? 0x80008000u : 0u;

    WorkFetcher wf;
    wf.init();
    int seq, lev, head;
    while (wf.next(p.hm, p.hdr, p.cursors, p.items, slot, seq, lev, head)) {
        ++n_done;
        const int row0 = p.cu[seq], L = p.cu[seq + 1] - row0;
        const int q0 = (lev - 1) * kFwdBM;
        const int kv_end = min(L, q0 + kFwdBM);
        const int n_kt = (kv_end + kFwdBN - 1) / kFwdBN;
        const int g = head / G;
        const int wrow0 = q0 + 32 * wave;                 // first query row of this wave
        const int qrow = wrow0 + l32;
        const bool qvalid = qrow < L;
        // K/V rows [0, kv_end) of this sequence and KV head; reads past them return zero
        const uint32_t kv_bytes = (uint32_t)(kv_end - 1) * (uint32_t)kv_stride * 2 + kRowBytes;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc(p.k + (int64_t)row0 * kv_stride + (int64_t)g * kHeadDim, kv_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc(p.v + (int64_t)row0 * kv_stride + (int64_t)g * kHeadDim, kv_bytes);

        bf16x8 qf[8];
        {
            const uint16_t* qp = p.q + (int64_t)(row0 + qrow) * q_stride + (int64_t)head * kHeadDim + 8 * half;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (qvalid) v = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
                qf[ks] = as_bf16x8(v ^ sign_flip);
            }
        }
        f32x16 acc_o[4];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
        float m_run = -INFINITY, l_run = 0.f;

        mk.load(rk, 0);
        mv.load(rv, 0);
        mk.store(smem);
        mv.store(smem + kFwdTileBytes);
        __syncthreads();
        // one tile step on LDS buffer BUF (compile-time, so that fragment reads are base+immediate)
        auto step = [&](auto buf_tag, int kt) {
            constexpr int BUF = decltype(buf_tag)::value;
            const char* Kt = smem + BUF * 2 * kFwdTileBytes;
            const char* Vt = Kt + kFwdTileBytes;
            const bool more = kt + 1 < n_kt;
#ifndef HYD_ABL_NOSTAGE
            if (more) {
                mk.load(rk, (uint32_t)(kt + 1) * tile_bytes);
                mv.load(rv, (uint32_t)(kt + 1) * tile_bytes);
            }
#endif
            const int key0 = kt * kFwdBN;
            if (key0 <= wrow0 + 31) {                     // some key of the tile is visible to the wave
                if (key0 + kFwdBN - 1 > wrow0)
                    fwd_tile<true>(Kt, Vt, fa, qf, acc_o, m_run, l_run, scale_log2, key0, qrow, half);
                else
                    fwd_tile<false>(Kt, Vt, fa, qf, acc_o, m_run, l_run, scale_log2, key0, qrow, half);
            }
#ifndef HYD_ABL_NOSTAGE
            if (more) {
                char* Kn = smem + (BUF ^ 1) * 2 * kFwdTileBytes;
                mk.store(Kn);
                mv.store(Kn + kFwdTileBytes);
            }
#endif
#ifndef HYD_ABL_NOBARRIER_INLOOP
            __syncthreads();
#endif
        };
        for (int kt = 0; kt < n_kt; kt += 2) {
            step(std::integral_constant<int, 0>{}, kt);
            if (kt + 1 < n_kt) step(std::integral_constant<int, 1>{}, kt + 1);
        }
        // epilogue: normalise, write O (bf16) and LSE (natural log)
        const float l_tot = l_run + shfl_xor32(l_run);
        const float inv = 1.f / l_tot;
        if (qvalid) {
            uint16_t* op = p.o + (int64_t)(row0 + qrow) * q_stride + (int64_t)head * kHeadDim + 4 * half;
#pragma unroll
            for (int db = 0; db < 4; ++db) {
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    u32x2 w = {pack_bf16(acc_o[db][4 * rq] * inv, acc_o[db][4 * rq + 1] * inv),
                               pack_bf16(acc_o[db][4 * rq + 2] * inv, acc_o[db][4 * rq + 3] * inv)};
                    *reinterpret_cast<u32x2*>(op + 32 * db + 8 * rq) = w;
                }
            }
            if (half == 0)
                p.lse[(int64_t)head * p.T + row0 + qrow] =
                    (m_run + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
        }
    }
    trace_write(p.tr, 0, t_start, n_done);
}

}  // namespace hyd
