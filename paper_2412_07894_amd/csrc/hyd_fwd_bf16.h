// bf16 forward kernel: block-diagonal causal flash-style tile loop on MFMA with fp32 accumulation.
//
// Work item = (sequence, 256-row query tile, query head).  A workgroup has 4 waves, one per SIMD;
// wave w owns query rows 64w..64w+63 of the tile as two 32-row blocks X and Y for the whole item,
// so the online softmax never crosses waves.  K and V tiles of 64 keys are staged through LDS
// (double buffered, one barrier per tile) and shared by the 4 waves.  Every K or V fragment read
// from LDS feeds two MFMAs (block X and block Y): LDS bandwidth, not the MFMA pipe, is what a
// one-block-per-wave layout runs out of first on this chip.
//
// Orientation.  Scores are computed transposed, S^T[key][q] = K Q^T, so that in the accumulator
// lane map (see mfma32) a lane owns ONE query row (column l%32) and 16 keys per 32-key block:
// the row maximum and row sum are in-lane reductions plus one exchange with the other half of
// the wave, and the softmax statistics m, l and the rescale factor are per-lane scalars.  The
// probabilities then feed the second product O^T[d][q] = V^T P^T directly as the B operand
// (contraction index = key = accumulator row), while V^T fragments come out of the row-major V
// tile with the transposing LDS read.
//
// Causality.  Tiles are 64 keys and a wave's rows start at a multiple of 64, so a wave meets
// exactly one partly masked tile, its diagonal tile (key0 == first row of the wave); in it block
// X sees only the first 32 keys (masked along the diagonal) and block Y sees the first 32 keys
// in full and the last 32 masked along the diagonal.  Every processed tile holds at least one
// visible key for every row, so the running maximum is finite from the first tile on.
#pragma once
#include <type_traits>

#include "hyd_sched.h"

namespace hyd {

constexpr int kFwdBM = 256, kFwdBN = 64, kFwdThreads = 256;
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

// Online-softmax update of one 32-row block over NKB 32-key score blocks; the last block is
// masked along the diagonal when DIAG (key index within the block > row index within the block).
// Produces the bf16 probabilities as B fragments pk[kb][0..7] and updates m, l and the output
// accumulators' scale.
template <int NKB, bool DIAG>
__device__ __forceinline__ void softmax_block(f32x16 (&s)[2], float& m_run, float& l_run, f32x16 (&acc)[4],
                                              float scale_log2, int krel, uint32_t (&pk)[2][8]) {
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float x = s[kb][r];
            if (DIAG && kb == NKB - 1) {
                if (8 * (r >> 2) + (r & 3) + krel > 0) x = -INFINITY;
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
            for (int r = 0; r < 16; ++r) acc[db][r] *= alpha;
        m_run = m_new;
    }
    float lsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            float t0 = __builtin_fmaf(s[kb][r], scale_log2, -m_run);
            float t1 = __builtin_fmaf(s[kb][r + 1], scale_log2, -m_run);
            if (DIAG && kb == NKB - 1) {
                if (8 * (r >> 2) + (r & 3) + krel > 0) t0 = -INFINITY;
                if (8 * (r >> 2) + (r & 3) + 1 + krel > 0) t1 = -INFINITY;
            }
            const float p0 = __builtin_amdgcn_exp2f(t0), p1 = __builtin_amdgcn_exp2f(t1);
            lsum += p0 + p1;
            pk[kb][r >> 1] = pack_bf16(p0, p1);
        }
    }
    l_run += lsum;
}

__device__ __forceinline__ bf16x8 p_frag(const uint32_t (&pk)[2][8], int b) {
    u32x4 v = {pk[b >> 1][4 * (b & 1) + 0], pk[b >> 1][4 * (b & 1) + 1], pk[b >> 1][4 * (b & 1) + 2],
               pk[b >> 1][4 * (b & 1) + 3]};
    return as_bf16x8(v);
}

// One 64-key tile for both row blocks of a wave.
template <bool DIAG>
__device__ __forceinline__ void fwd_tile(const char* Kt, const char* Vt, const FragAddr& fa,
                                         const bf16x8 (&qf)[2][8], f32x16 (&acc_o)[2][4], float (&m_run)[2],
                                         float (&l_run)[2], float scale_log2, int krel) {
    f32x16 s[2][2];       // [row block][key block]
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[qb][kb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const bf16x8 a = frag_row(Kt, fa, kb, ks);
            // block X never sees keys 32..63 of its diagonal tile
            if (!(DIAG && kb == 1)) s[0][kb] = mfma32(a, qf[0][ks], s[0][kb]);
            s[1][kb] = mfma32(a, qf[1][ks], s[1][kb]);
        }
    }
    uint32_t pk[2][2][8];
    if (DIAG) softmax_block<1, true>(s[0], m_run[0], l_run[0], acc_o[0], scale_log2, krel, pk[0]);
    else softmax_block<2, false>(s[0], m_run[0], l_run[0], acc_o[0], scale_log2, krel, pk[0]);
    softmax_block<2, DIAG>(s[1], m_run[1], l_run[1], acc_o[1], scale_log2, krel, pk[1]);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const bf16x8 a = frag_col(Vt, fa, b, db);
            if (!(DIAG && b >= 2)) acc_o[0][db] = mfma32(a, p_frag(pk[0], b), acc_o[0][db]);
            acc_o[1][db] = mfma32(a, p_frag(pk[1], b), acc_o[1][db]);
        }
    }
}

__global__ void __launch_bounds__(kFwdThreads, 1) hyd_fwd_bf16_kernel(FwdParams p) {
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
    const int krel = 4 * half - l32;          // (key index in block) - (row index in block) offset

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
        const int wrow0 = q0 + 64 * wave;                 // first query row of this wave
        // K/V rows [0, kv_end) of this sequence and KV head; reads past them return zero
        const uint32_t kv_bytes = (uint32_t)(kv_end - 1) * (uint32_t)kv_stride * 2 + kRowBytes;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc(p.k + (int64_t)row0 * kv_stride + (int64_t)g * kHeadDim, kv_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc(p.v + (int64_t)row0 * kv_stride + (int64_t)g * kHeadDim, kv_bytes);

        bf16x8 qf[2][8];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int qrow = wrow0 + 32 * qb + l32;
            const uint16_t* qp = p.q + (int64_t)(row0 + qrow) * q_stride + (int64_t)head * kHeadDim + 8 * half;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (qrow < L) v = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
                qf[qb][ks] = as_bf16x8(v ^ sign_flip);
            }
        }
        f32x16 acc_o[2][4];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[qb][db][r] = 0.f;
        float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

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
            if (more) {
                mk.load(rk, (uint32_t)(kt + 1) * tile_bytes);
                mv.load(rv, (uint32_t)(kt + 1) * tile_bytes);
            }
            const int key0 = kt * kFwdBN;
            if (wrow0 >= L) {
                // no row of this wave exists: it only helps with staging
            } else if (key0 < wrow0) fwd_tile<false>(Kt, Vt, fa, qf, acc_o, m_run, l_run, scale_log2, krel);
            else if (key0 == wrow0) fwd_tile<true>(Kt, Vt, fa, qf, acc_o, m_run, l_run, scale_log2, krel);
            if (more) {
                char* Kn = smem + (BUF ^ 1) * 2 * kFwdTileBytes;
                mk.store(Kn);
                mv.store(Kn + kFwdTileBytes);
            }
            __syncthreads();
        };
        for (int kt = 0; kt < n_kt; kt += 2) {
            step(std::integral_constant<int, 0>{}, kt);
            if (kt + 1 < n_kt) step(std::integral_constant<int, 1>{}, kt + 1);
        }
        // epilogue: normalise, write O (bf16) and LSE (natural log)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int qrow = wrow0 + 32 * qb + l32;
            const float l_tot = l_run[qb] + shfl_xor32(l_run[qb]);
            const float inv = 1.f / l_tot;
            if (qrow < L) {
                uint16_t* op = p.o + (int64_t)(row0 + qrow) * q_stride + (int64_t)head * kHeadDim + 4 * half;
#pragma unroll
                for (int db = 0; db < 4; ++db) {
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        u32x2 w = {pack_bf16(acc_o[qb][db][4 * rq] * inv, acc_o[qb][db][4 * rq + 1] * inv),
                                   pack_bf16(acc_o[qb][db][4 * rq + 2] * inv, acc_o[qb][db][4 * rq + 3] * inv)};
                        *reinterpret_cast<u32x2*>(op + 32 * db + 8 * rq) = w;
                    }
                }
                if (half == 0)
                    p.lse[(int64_t)head * p.T + row0 + qrow] =
                        (m_run[qb] + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
            }
        }
    }
    trace_write(p.tr, 0, t_start, n_done);
}

}  // namespace hyd
