// bf16 backward kernels: row statistics and fp16 operand copies, dK/dV, and dQ.  No atomics on
// results: every output element has exactly one producing wave with a fixed summation order, so
// results are bitwise reproducible (the one atomic, a maximum over |dO|, does not depend on order).
//
// Arithmetic.  The four products that consume a factor formed in registers (dV = P^T dO,
// dK = dS^T Q, dQ = dS K) and the products next to them run on the fp16 MFMA: P and dS keep 11
// significant bits instead of the 8 that bf16 would leave them, which is what an absolute error
// bar of 2e-2 on gradients of size 4-8 needs (their own rounding to bf16 already takes 1.6e-2 of
// it).  Every bf16 input converts to fp16 exactly as long as its magnitude lies in [2^-14, 65504];
// dO, whose scale is arbitrary (it is linear in the loss), is brought into that range by powers
// of two: one per tensor for dK/dV (sums over rows need a common scale), one per row for dQ
// (applied to the row's dO and D when the dQ kernel takes them into registers), both undone when
// the results are written.  Powers of two are exact, so the gradients follow a power-of-two scale
// of dO bit for bit.  The fp16 copies of Q, K and dO that the tile loops stream are written once per call
// into the workspace.
//
// Fragment convention (see hyd_device.h): an MFMA operand fragment is "lane <-> one index, 8
// register slots <-> contraction index" and can be used as the A or the B operand alike; the
// product D[a][b] then has the A fragment's lane index as its row and B's as its column, and an
// accumulator in turn is a fragment whose lane index is the column and whose slots are rows.
#pragma once
#include <type_traits>

#include "hyd_sched.h"

namespace hyd {

constexpr float kLog2e = 1.44269504088896340736f;

// Power-of-two exponent k that brings a magnitude (given by the 15 low bits of its bf16 pattern)
// into [1, 2): |x| * 2^k.  Zero, subnormal, infinite and NaN magnitudes give 0; |k| <= kMaxShift
// keeps 2^k, 2^-k and P * 2^k inside fp32.
constexpr int kMaxShift = 100;
__device__ __forceinline__ int shift_of(uint32_t abs_bf16) {
    const int e = (int)(abs_bf16 >> 7);                  // biased exponent
    if (e == 0 || e == 255) return 0;
    const int k = 127 - e;
    return k > kMaxShift ? kMaxShift : (k < -kMaxShift ? -kMaxShift : k);
}
__device__ __forceinline__ float pow2i(int k) { return __uint_as_float((uint32_t)(127 + k) << 23); }

// Row statistics and scratch of the backward, all in the caller's workspace.
struct BwdScratch {
    float* Dq;          // [Hq][T]  -D,  D = rowsum(dO * O)                          (dQ kernel)
    float* kqmul;       // [Hq][T]  2^-kq, kq = shift_of(row max |dO|)               (dQ kernel: row scale and its inverse)
    float* lse2;        // [Hq][T]  -LSE * log2(e)                                   (both kernels)
    float* Dkv;         // [Hq][T]  -D * 2^kg, kg = shift_of(max |dO| of the tensor) (dK/dV kernel; written by dQ)
    uint32_t* absmax;   // max over dO of the 15-bit magnitude pattern; zeroed by the schedule prelude
    uint16_t* q16;      // [T][Hq][d]  fp16 copy of Q          (written by the dQ kernel, read by dK/dV)
    uint16_t* do16;     // [T][Hq][d]  fp16 copy of dO * 2^kg  (written by the dQ kernel, read by dK/dV)
    uint16_t* k16;      // [T][Hkv][d] fp16 copy of K          (written by the statistics pass)
};

// ---------------------------------------------------------------------------------------------
// One pass over O, dO and K before the tile kernels (16 lanes per row, kStatTok = 32 tokens per workgroup):
// the row statistics above except Dkv, the tensor's largest |dO|, and the fp16 copy of K.  A
// workgroup walks the rows of its tokens in memory order and collects their statistics in LDS, so
// that the [Hq][T] vectors are written in runs of kStatTok consecutive floats.  The statistics are
// stored NEGATED: the form in which the two backward kernels consume them
// (P = exp2(s * scale * log2(e) + (-LSE2)), dS = P * (dP + (-D))), so that dK/dV can use -D as the
// initial value of its dP accumulator.  (The fp16 copies of Q and dO and Dkv are written by the dQ
// kernel, which has those rows in LDS anyway.)
// ---------------------------------------------------------------------------------------------
// tokens per workgroup: 32, fewer with very many heads so that the statistics stay within 32 KB of LDS
inline int rowstats_tokens(int hq) { const int t = 4096 / (hq > 0 ? hq : 1); return t > 32 ? 32 : (t < 1 ? 1 : t); }
inline size_t rowstats_lds(int hq) { return sizeof(float) * 2 * (size_t)hq * rowstats_tokens(hq); }

template <int HD = kHeadDim>
__global__ void __launch_bounds__(256) hyd_bwd_rowstats_bf16_kernel(const uint16_t* __restrict__ o,
                                                                   const uint16_t* __restrict__ d_o,
                                                                   const float* __restrict__ lse,
                                                                   const uint16_t* __restrict__ k,
                                                                   BwdScratch sc, int T, int hq, int hkv, int kStatTok) {
    extern __shared__ float st[];                  // [2][hq][kStatTok]: -D, kq
    const int t0 = blockIdx.x * kStatTok;
    const int nt = min(kStatTok, T - t0);
    const int grp = threadIdx.x >> 4, c = threadIdx.x & 15;
    const bool lane_on = HD == kHeadDim || c < HD / 8;
    uint32_t gmax = 0;
    for (int r = grp; r < nt * hq; r += 16) {      // row r of the block = (token t0 + r / hq, head r % hq)
        const int64_t at = ((int64_t)t0 * hq + r) * HD + c * 8;
        float acc = 0.f;
        uint32_t amax = 0;
        if (lane_on) {
            const u32x4 a = *reinterpret_cast<const u32x4*>(o + at);
            const u32x4 b = *reinterpret_cast<const u32x4*>(d_o + at);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc += bf16_lo(a[e]) * bf16_lo(b[e]) + bf16_hi(a[e]) * bf16_hi(b[e]);
                amax = max(amax, max(b[e] & 0x7fffu, (b[e] >> 16) & 0x7fffu));
            }
        }
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {
            acc += __shfl_xor(acc, m, 64);
            amax = max(amax, (uint32_t)__shfl_xor((int)amax, m, 64));
        }
        if (c == 0) {
            const int tl = r / hq, h = r - tl * hq;
            st[h * kStatTok + tl] = -acc;
            st[(hq + h) * kStatTok + tl] = (float)shift_of(amax);
        }
        gmax = max(gmax, amax);
    }
    for (int r = grp; r < nt * hkv; r += 16) {     // the K rows of the same tokens
        if (lane_on) {
            const int64_t at = ((int64_t)t0 * hkv + r) * HD + c * 8;
            const u32x4 x = *reinterpret_cast<const u32x4*>(k + at);
            u32x4 x16;
#pragma unroll
            for (int e = 0; e < 4; ++e) x16[e] = bf16x2_to_f16x2(x[e]);
            *reinterpret_cast<u32x4*>(sc.k16 + at) = x16;
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < hq * kStatTok; idx += 256) {
        const int h = idx / kStatTok, tl = idx % kStatTok;
        if (tl < nt) {
            const int64_t at = (int64_t)h * T + t0 + tl;
            const float l2 = -lse[at] * kLog2e, kq = st[(hq + h) * kStatTok + tl];
            sc.Dq[at] = st[idx];
            sc.kqmul[at] = pow2i(-(int)kq);
            sc.lse2[at] = l2;
        }
    }
    // the tensor's maximum: one atomic per wave at most, and none once the stored value has caught
    // up (the plain read only filters; the atomic decides)
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) gmax = max(gmax, (uint32_t)__shfl_xor((int)gmax, m, 64));
    if ((threadIdx.x & 63) == 0 && gmax > __hip_atomic_load(sc.absmax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(sc.absmax, gmax);
}

struct BwdParams {
    const uint16_t* q; const uint16_t* v; const uint16_t* d_o;     // the caller's bf16 Q, V and dO (dQ kernel; dK/dV: V only)
    BwdScratch sc;
    uint16_t* dq; uint16_t* dk; uint16_t* dv;
    int T, hq, hkv;
    float scale, scale_log2;
    const int* hdr; int* cursors; const int* items;
    HeadMap hm;
    WgTrace tr;
    const int32_t* ranges;            // range variants only: per sequence (q_begin, q_end, kv_begin, kv_end)
    const double* rope_tab;           // NULL, or the rotary frequency table: the dQ kernel rotates Q as it picks it up
                                      // (the fp16 copy it writes is the rotated Q) and turns dQ back before writing it
};

// ---------------------------------------------------------------------------------------------
// dQ.  Work item = (sequence, query tile of 256 rows, query head); wave w of 8 owns rows 32w..32w+31.
// Same orientation, K/V ring and causal structure as the forward kernel: S^T[key][q] = K Q^T and
// dP^T[key][q] = V dO^T put one query row in each lane, so LSE_i and D_i are per-lane scalars;
// dS^T then is the B operand of dQ^T[d][q] = K^T dS^T, with K^T fragments from the transposing
// LDS read of the same K tile.  The K tiles are the fp16 copy (score and dQ products on the fp16
// MFMA, Q rows from the fp16 copy too); V tiles and dO rows are the caller's bf16 tensors (dP on
// the bf16 MFMA, exact inputs either way).  The row's dO and D are multiplied by 2^kq, the power
// of two that brings the row's largest |dO| into [1, 2), as they are taken into registers, so
// dS = P (dP - D) is formed for the scaled row (inside fp16's range whatever the scale of the
// loss) and dQ is scaled back by 2^-kq when it is written.
// This kernel runs BEFORE dK/dV and, having every Q and dO row of its item in LDS once, also writes
// what that kernel streams: the fp16 copies of Q and of dO * 2^kg, and -D * 2^kg.
// ---------------------------------------------------------------------------------------------
constexpr int kDqWaves = 8;
constexpr int kDqBM = 32 * kDqWaves, kDqBN = 64, kDqThreads = 64 * kDqWaves;
constexpr int kDqStages = 3;
constexpr int kDqTileBytes = kDqBN * kRowBytes;
constexpr int kDqStageBytes = 2 * kDqTileBytes;
// Staging of the item's Q and dO rows (direct-to-LDS loads of whole rows, as in the forward
// kernel): Q in a region of its own, dO in ring stages 1 and 2, which no K/V tile needs before
// the rows have been taken into registers.  The work slot shares the first bytes of the Q region:
// it is idle while rows are staged (a barrier separates its last read from those loads).
constexpr int kDqQxOff = kDqStages * kDqStageBytes;
constexpr int kDqLds = kDqQxOff + kDqBM * kRowBytes;                  // 160 KB: all of a CU's LDS

typedef __attribute__((address_space(3))) void lds_void_b;

// One 32-key block (rows 32*kb.. of the K and V tiles) for the 32 rows of a wave.  `k0`: key index
// minus row index of the block's first key for this lane's row if the block needs masking, else a
// value that masks nothing.
// D: head dimension (128 or 64).
template <int D>
__device__ __forceinline__ void dq_block(int Kt, int Vt, const FragAddr& fa, int kb,
                                         const bf16x8 (&qf)[D / 16], const bf16x8 (&dof)[D / 16], f32x16 (&acc)[D / 32],
                                         float scale_log2, float lse2, float Dq, bool mask, int krel) {
    // lse2 and Dq hold -LSE2 and -D * 2^kq of the lane's row; qf and the K tile are fp16, dof (dO * 2^kq) and the V tile bf16
    constexpr int NK = D / 16, NDB = D / 32;
    // instruction order pinned with scheduling fences (see the forward kernel)
    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }

    {
        // fragment i < NK: K, contraction step i; i >= NK: V, step i - NK; reads run kAhead ahead
        constexpr int kAhead = 4;
        bf16x8 f[kAhead];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) f[i] = frag_row(i < NK ? Kt : Vt, fa, kb, i % NK);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2 * NK; ++i) {
            if (i == NK && mask) {                // the score block is complete; hidden keys: P = exp2(-inf) = 0
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (8 * (r >> 2) + (r & 3) + krel > 0) s[r] = -INFINITY;
            }
            if (i < NK) s = mfma32h(f[i % kAhead], qf[i], s);
            else dp = mfma32(f[i % kAhead], dof[i - NK], dp);
            if (i + kAhead < 2 * NK) f[i % kAhead] = frag_row(i + kAhead < NK ? Kt : Vt, fa, kb, (i + kAhead) % NK);
            if (i >= NK) {                        // the exponentials of the finished score block run under the dP product
#pragma unroll
                for (int e = 0; e < 16 / NK; ++e) {
                    const int r = (16 / NK) * (i - NK) + e;
                    s[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, lse2));    // s becomes P in place
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    constexpr int kCAhead = 4;
    LdsQueue lq{0};
    ColFrag cf[kCAhead];                      // K^T fragments for the dQ product, requested early
#pragma unroll
    for (int i = 0; i < kCAhead && i < 2 * NDB; ++i) issue_col(lq, cf[i], Kt, fa, 2 * kb + i / NDB, i % NDB);
    __builtin_amdgcn_sched_barrier(0);
    auto ds_pair = [&](int j) -> uint32_t {   // scores 2j, 2j+1 of the 16 a lane holds
        const int r = 2 * j;
        return pack_f16(s[r] * (dp[r] + Dq), s[r + 1] * (dp[r + 1] + Dq));      // s holds P by now; dp and Dq carry 2^kq
    };
    u32x4 dcur, dnxt;
#pragma unroll
    for (int e = 0; e < 4; ++e) dcur[e] = ds_pair(e);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 2 * NDB; ++i) {       // i = NDB*b2 + db
        const int b2 = i / NDB, db = i % NDB;
        acc[db] = mfma32h(lds_wait(lq, cf[i % kCAhead]), as_bf16x8(dcur), acc[db]);
        if (i + kCAhead < 2 * NDB) issue_col(lq, cf[i % kCAhead], Kt, fa, 2 * kb + (i + kCAhead) / NDB, (i + kCAhead) % NDB);
        if (b2 == 0) {
#pragma unroll
            for (int e = 0; e < 4 / NDB; ++e) dnxt[(4 / NDB) * db + e] = ds_pair(4 + (4 / NDB) * db + e);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (i == NDB - 1) dcur = dnxt;
    }
}

// R: range variant (see the forward kernel): query tiles outside the query range are skipped,
// the tile loop covers the key range only, dQ holds that key range's contribution.
template <bool R, int D = kHeadDim>
__global__ void __launch_bounds__(kDqThreads, 1) hyd_bwd_dq_bf16_kernel(BwdParams p) {
    static_assert(D == 128 || D == 64, "head dimension");
    constexpr int kRowB = D * 2;                                      // bytes of a row in global memory
    static_assert(kDqBM == 256 && kDqStages == 3, "the Q / dO staging assumes a 256-row tile and a 3-stage ring");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int* slot = reinterpret_cast<int*>(smem + kDqQxOff);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int G = p.hq / p.hkv;
    const int64_t q_stride = (int64_t)p.hq * D, kv_stride = (int64_t)p.hkv * D;
    const uint32_t kv_stride_b = (uint32_t)kv_stride * 2, q_stride_b = (uint32_t)q_stride * 2;
    const unsigned long long t_start = p.tr.rec ? wall_clock64() : 0ull;
    unsigned long long n_done = 0;

    FragAddr fa;
    fa.init(lane, smem);
    const int dma_row = 4 * wave + (lane >> 4);
    const uint32_t dma_voff = dma_lane_voff<D>(dma_row, lane, kv_stride_b);
    const uint32_t dma_voff_q = dma_lane_voff<D>(dma_row, lane, q_stride_b);
    const uint32_t tile_bytes = kDqBN * kv_stride_b;
    // this wave's 32 rows inside a staged 256-row block, and its private 8 KB of the ring for dQ
    const int row_stage = wave * 32 * kRowBytes;
    const uint32_t o_stage = (uint32_t)(uintptr_t)(lds_char*)smem + (uint32_t)row_stage;
    // scale * s = |scale| * (-s): a negative scale flips the sign bits of the Q fragments, which
    // only the score product reads; a zero scale becomes an epsilon so that -inf * scale = -inf
    const float scale_log2 = fmaxf(fabsf(p.scale_log2), 1e-30f);
    const uint32_t sign_flip = p.scale_log2 < 0.f ? 0x80008000u : 0u;
    const float up = pow2i(shift_of(*p.sc.absmax));                   // 2^kg
    const bool wave_first_half = half == 0;                           // both halves of a wave hold the same rows

    WorkFetcher wf;
    WorkItem wi;
    bool have = wf.first(p.hm, p.hdr, p.cursors, p.items, slot, wi);
    while (have) {
        ++n_done;
        __syncthreads();                                  // everybody has read the work slot: its bytes may be overwritten
        const int lev = wi.lev, head = wi.head, row0 = wi.row0, L = wi.len;
        const int q0 = (lev - 1) * kDqBM;
        int Lq = L, kb = 0, kcap = L;                     // query rows [.., Lq), keys [kb, kcap)
        if (R) {
            const i32x4 rg = *reinterpret_cast<const i32x4*>(p.ranges + 4 * wi.seq);
            Lq = min(L, rg[1]); kb = max(rg[2], 0); kcap = min(L, rg[3]);
            if (q0 < rg[0] || q0 >= Lq) {
                have = wf.next(p.hm, p.cursors, p.items, slot, wi);
                continue;
            }
        }
        const int kv_end = min(kcap, q0 + kDqBM);
        const int n_kt = (kv_end + kDqBN - 1) / kDqBN;
        const int t_lo = R ? kb / kDqBN : 0;
        const int g = head / G;
        const int wrow0 = q0 + 32 * wave;
        const int qrow = wrow0 + l32;
        const bool qvalid = qrow < Lq;
        const bool active = wrow0 < Lq;
        if (R && kv_end <= kb) {                          // no key of the range is visible: dQ = 0
            if (qvalid) {
                uint16_t* op = p.dq + (int64_t)(row0 + qrow) * q_stride + (int64_t)head * D + 4 * half;
                const u32x2 z = {0u, 0u};
#pragma unroll
                for (int i = 0; i < D / 8; ++i) *reinterpret_cast<u32x2*>(op + 8 * i) = z;
            }
            have = wf.next(p.hm, p.cursors, p.items, slot, wi);
            continue;
        }
        const int td = wrow0 / kDqBN;                     // this wave's diagonal (= last) tile
        const int diag_kb = (wrow0 % kDqBN) / 32;         // its diagonal block within that tile
        const uint32_t kv_bytes = (uint32_t)(kv_end - 1) * kv_stride_b + kRowB;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc(p.sc.k16 + (int64_t)row0 * kv_stride + (int64_t)g * D, kv_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc(p.v + (int64_t)row0 * kv_stride + (int64_t)g * D, kv_bytes);
        auto dma_tile = [&](int t, int stage) {
            char* dst = smem + stage * kDqStageBytes + 4 * wave * kRowBytes;
#pragma unroll
            for (int j = 0; j < 16 / kDqWaves; ++j) {
                const uint32_t soff = (uint32_t)t * tile_bytes + (uint32_t)(j * kDqWaves * 4) * kv_stride_b;
                char* d = dst + j * kDqWaves * 4 * kRowBytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lds_void_b*)d, 16, dma_voff, soff, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_void_b*)(d + kDqTileBytes), 16, dma_voff, soff, 0, 0);
            }
        };
        dma_tile(t_lo, 0);
        {   // rows q0 .. q0+255 of Q and dO of this head; rows past the query range read as zeros
            const uint32_t q_bytes = (uint32_t)(min(Lq - q0, kDqBM) - 1) * q_stride_b + kRowB;
            const int64_t off = (int64_t)(row0 + q0) * q_stride + (int64_t)head * D;
            dma_rows<kDqWaves>(make_rsrc(p.q + off, q_bytes), smem + kDqQxOff, [](int j) { return j * kDqTileBytes; },
                               kDqBM / 64, q_stride_b, wave, dma_voff_q);
            dma_rows<kDqWaves>(make_rsrc(p.d_o + off, q_bytes), smem + kDqStageBytes, [](int j) { return j * kDqTileBytes; },
                               kDqBM / 64, q_stride_b, wave, dma_voff_q);
        }
        float lse2 = 0.f, Dq = 0.f, unshift = 0.f;
        if (qvalid) {
            lse2 = p.sc.lse2[(int64_t)head * p.T + row0 + qrow];
            Dq = p.sc.Dq[(int64_t)head * p.T + row0 + qrow];
            unshift = p.sc.kqmul[(int64_t)head * p.T + row0 + qrow];
            if (wave_first_half) p.sc.Dkv[(int64_t)head * p.T + row0 + qrow] = Dq * up;
        }
        // 2^kq, the exact reciprocal of the power of two 2^-kq; rows past the range keep 1
        const float shift = qvalid ? __uint_as_float((254u << 23) - __float_as_uint(unshift)) : 1.f;
        Dq *= shift;
        f32x16 acc[D / 32];
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
        __syncthreads();                                  // tile t_lo and the Q / dO rows have landed
        bf16x8 qf[D / 16], dof[D / 16];
        {
            u32x4 a[D / 16], b[D / 16];
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                a[ks] = *(lds_u32x4*)(uintptr_t)(fa.row[ks] + (uint32_t)(kDqQxOff + row_stage));
                b[ks] = *(lds_u32x4*)(uintptr_t)(fa.row[ks] + (uint32_t)(kDqStageBytes + row_stage));
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);           // lgkmcnt(0)
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(a[ks]), "+v"(b[ks]));      // the reads stay on this side of the barrier
            // Q -> fp16, rotated first if the call asks for it (position = local row: reset per sequence)
            if (p.rope_tab) {
                rope_row_frags<D, true>(a, p.rope_tab, qrow, half);
            } else {
#pragma unroll
                for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[ks][e] = bf16x2_to_f16x2(a[ks][e]);
            }
            // What the dK/dV kernel streams: the fp16 Q rows and dO * 2^kg.  Each wave puts its 32 rows
            // back where it took them from (nobody else touches those bytes) and sends them out from
            // there in 16-byte pieces of whole rows: four whole rows per store instruction.
            typedef __attribute__((address_space(3))) u32x4 lds_u32x4_w;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                u32x4 s16;
#pragma unroll
                for (int e = 0; e < 4; ++e) s16[e] = bf16x2_to_f16x2(b[ks][e], up);
                *(lds_u32x4_w*)(uintptr_t)(fa.row[ks] + (uint32_t)(kDqQxOff + row_stage)) = a[ks];
                *(lds_u32x4_w*)(uintptr_t)(fa.row[ks] + (uint32_t)(kDqStageBytes + row_stage)) = s16;
            }
            // (the lane index is laundered so that these addresses are formed here: hoisted above the
            // tile loop as lane constants they would occupy some 20 registers through it)
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int cr = ln >> 4, ch = ln & 15;
            const uint32_t wbase = (uint32_t)(uintptr_t)(lds_char*)smem + (uint32_t)(row_stage + cr * kRowBytes);
            const int64_t goff = (int64_t)(row0 + wrow0 + cr) * q_stride + (int64_t)head * D + ch * 8;
#pragma unroll
            for (int which = 0; which < 2; ++which) {
                uint16_t* dst = (which ? p.sc.do16 : p.sc.q16) + goff;
                u32x4 x[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)                 // row cr + 4 i of the wave: swz = (cr << 2) | (i & 3)
                    x[i] = *(lds_u32x4*)(uintptr_t)(wbase + (uint32_t)((which ? kDqStageBytes : kDqQxOff) + 4 * i * kRowBytes +
                                                                      ((ch ^ ((cr << 2) | (i & 3))) << 4)));
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (wrow0 + cr + 4 * i < Lq && (D == kHeadDim || ch < D / 8))
                        *reinterpret_cast<u32x4*>(dst + (int64_t)(4 * i) * q_stride) = x[i];
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);           // lgkmcnt(0): the staging areas have been read
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                qf[ks] = as_bf16x8(a[ks] ^ sign_flip);
                // the row's dO times 2^kq (exact: a power of two, and the row's largest element lands in [1, 2))
#pragma unroll
                for (int e = 0; e < 4; ++e) b[ks][e] = pack_bf16(bf16_lo(b[ks][e]) * shift, bf16_hi(b[ks][e]) * shift);
                dof[ks] = as_bf16x8(b[ks]);
            }
        }
        __builtin_amdgcn_s_barrier();                     // stages 1 and 2 may take K/V tiles now
        if (t_lo + 1 < n_kt) dma_tile(t_lo + 1, 1);

        auto step = [&](auto stage_tag, int t) {
            constexpr int ST = decltype(stage_tag)::value;
            constexpr int Kt = ST * kDqStageBytes, Vt = Kt + kDqTileBytes;        // LDS offsets of the tiles
            // the loads run two tiles ahead: tile t+1 was requested one step ago and precedes this
            // step's loads in the (in-order) vmcnt queue
            constexpr int ST2 = (ST + 2) % kDqStages;
            constexpr int kDmaPerTile = 2 * (16 / kDqWaves);
            const bool more2 = t + 2 < n_kt;
            if (more2) dma_tile(t + 2, ST2);
            if (active && t <= td) {
                const bool diag = t == td;
                // key-minus-row offset of the masked block, formed from the tile index so that the
                // mask comparisons are not hoisted out of the tile loop into scalar registers
                const int krel = t * kDqBN + 32 * diag_kb + 4 * half - qrow;
                dq_block<D>(Kt, Vt, fa, 0, qf, dof, acc, scale_log2, lse2, Dq, diag && diag_kb == 0, krel);
                if (!(diag && diag_kb == 0))
                    dq_block<D>(Kt, Vt, fa, 1, qf, dof, acc, scale_log2, lse2, Dq, diag, krel);
            }
            if (more2) __builtin_amdgcn_s_waitcnt(0x0070 | (kDmaPerTile & 15));     // vmcnt(kDmaPerTile), lgkmcnt(0)
            else __builtin_amdgcn_s_waitcnt(0x0070);                                // vmcnt(0), lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
        };
        for (int t = t_lo; t < n_kt; t += 3) {
            step(std::integral_constant<int, 0>{}, t);
            if (t + 1 < n_kt) step(std::integral_constant<int, 1>{}, t + 1);
            if (t + 2 < n_kt) step(std::integral_constant<int, 2>{}, t + 2);
        }
        if (active && p.rope_tab) rope_acc_inverse<D>(acc, p.rope_tab, qrow, half);     // gradient of the UNROTATED Q
        if (active)         // dQ leaves through this wave's 8 KB of the ring (free now): whole rows per store
            store_rows_via_lds<D>(p.dq + (int64_t)(row0 + wrow0) * q_stride + (int64_t)head * D, q_stride, Lq - wrow0,
                               acc, p.scale * unshift, o_stage, lane);
        have = wf.next(p.hm, p.cursors, p.items, slot, wi);
    }
    trace_write(p.tr, 2, t_start, n_done);
}

// ---------------------------------------------------------------------------------------------
// dK/dV.  Work item = (sequence, 128-key tile, KV head).  A workgroup has 8 waves in 4 pairs; pair
// p owns keys 32p..32p+31 of the tile.  The two waves of a pair share a SIMD and split the four
// products of a (32 query rows x 32 keys) block by role, so that each wave needs half the
// accumulators (two waves fit one SIMD) and each hides the other's non-MFMA work:
//     role A (waves 0-3): S = Q K^T  -> P = exp2(S*scale - LSE2) -> hands P to its partner through
//                         LDS -> dV^T += dO^T P
//     role B (waves 4-7): dP' = dO V^T - D -> takes P -> dS = P dP' -> dK^T += Q^T dS
// -D of the block's rows is the INITIAL VALUE of role B's dP accumulator, read from the stage into
// the accumulator registers: the MFMA chain then delivers the factor of dS itself and the
// subtraction per element leaves the vector ALU (role A cannot do the same with -LSE2 without a
// pre-scaled K, whose rounding to bf16 costs a quarter more error in dK and dV).
// S[i][j] and dP[i][j] put one KEY in each lane (accumulator column) and query rows in the slots,
// so P and dS are directly the B fragments (contraction index = query row) of the second
// products, whose A fragments come from the transposing LDS read of the dO and Q tiles.  P crosses
// lane-to-lane (same accumulator layout on both sides) as fp16, the form in which role A's own
// dV product consumes it.  All four products run on the fp16 MFMA: the Q and dO tiles are the
// fp16 copies (dO scaled by 2^kg), K rows come from the fp16 copy, V rows are converted in
// registers once per item; dK and dV are scaled back by 2^-kg when they are written.
// Query tiles of 64 rows (Q, dO, LSE2, D) stream through a ring of 3 LDS stages by
// direct-to-LDS loads, for every query head of the KV group in turn, accumulating into the same
// registers.  One workgroup barrier per 32-row block: it publishes P and, every second block,
// the next tile.
// ---------------------------------------------------------------------------------------------
constexpr int kKvPairs = 4, kKvWaves = 2 * kKvPairs;
constexpr int kKvBN = 32 * kKvPairs, kKvBM = 64, kKvThreads = 64 * kKvWaves, kKvStages = 3;
constexpr int kKvTileBytes = kKvBM * kRowBytes;                       // 16 KB
constexpr int kKvStageBytes = 2 * kKvTileBytes + 2 * kKvBM * 4;       // Q, dO, LSE2, D
constexpr int kKvPBytes = 64 * 16 * 4;                                // P buffer of a block (64 lanes x 16 values; fp16 fills half)
constexpr int kKvPOff = kKvStages * kKvStageBytes;                    // P exchange: [pair][2][kKvPBytes]
constexpr int kKvLds = kKvPOff + kKvPairs * 2 * kKvPBytes + 64;

// R: range variant (see the forward kernel): key tiles outside the key range are skipped, the
// query tiles run over the query range only, dK / dV hold that query range's contribution.
template <bool R, int D = kHeadDim>
__global__ void __launch_bounds__(kKvThreads, 1) hyd_bwd_dkdv_bf16_kernel(BwdParams p) {
    static_assert(D == 128 || D == 64, "head dimension");
    constexpr int kRowB = D * 2;                                      // bytes of a row in global memory
    constexpr int NK = D / 16, NDB = D / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int* slot = reinterpret_cast<int*>(smem + kKvPOff + kKvPairs * 2 * kKvPBytes);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pair = wave & (kKvPairs - 1);
    const bool role_b = wave >= kKvPairs;
    const int l32 = lane & 31, half = lane >> 5;
    const int G = p.hq / p.hkv;
    const int64_t q_stride = (int64_t)p.hq * D, kv_stride = (int64_t)p.hkv * D;
    const uint32_t q_stride_b = (uint32_t)q_stride * 2;
    const unsigned long long t_start = p.tr.rec ? wall_clock64() : 0ull;
    unsigned long long n_done = 0;

    FragAddr fa;
    fa.init(lane, smem);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        fa.row[i] += role_b ? kKvTileBytes : 0;
        fa.col[i] += role_b ? 0 : kKvTileBytes;
    }
    const int dma_row = 4 * wave + (lane >> 4);
    const uint32_t dma_voff = dma_lane_voff<D>(dma_row, lane, q_stride_b);
    const uint32_t tile_bytes = kKvBM * q_stride_b;                   // one Q/dO tile in global memory
    // K and V rows of the item arrive by direct-to-LDS loads of whole rows (K in ring stage 2, V
    // in the P exchange area, both idle until the first step) and are taken into registers from
    // there; dK / dV leave through 8 KB of the (then free) ring per wave
    const uint32_t kv_stride_b = (uint32_t)kv_stride * 2;
    const uint32_t dma_voff_kv = dma_lane_voff<D>(dma_row, lane, kv_stride_b);
    const uint32_t kv_stage = (role_b ? kKvPOff : 2 * kKvStageBytes) + pair * 32 * kRowBytes - (role_b ? kKvTileBytes : 0);
    const uint32_t o_stage = (uint32_t)(uintptr_t)(lds_char*)smem + (uint32_t)(wave * 32 * kRowBytes);
    // a negative scale flips the sign bits of the K fragments, which only the score product reads;
    // a zero scale becomes an epsilon so that -inf * scale = -inf
    const float scale_log2 = fmaxf(fabsf(p.scale_log2), 1e-30f);
    const uint32_t sign_flip = p.scale_log2 < 0.f ? 0x80008000u : 0u;
    char* const pbuf = smem + kKvPOff + pair * 2 * kKvPBytes + lane * 8;      // + buf * kKvPBytes + q * 512
    const float unscale = pow2i(-shift_of(*p.sc.absmax));                     // 2^-kg

    WorkFetcher wf;
    WorkItem wi;
    bool have = wf.first(p.hm, p.hdr, p.cursors, p.items, slot, wi);
    while (have) {
        ++n_done;
        const int lev = wi.lev, g = wi.head, row0 = wi.row0, L = wi.len;
        const int n_tiles = (L + kKvBN - 1) / kKvBN;
        const int j0 = (n_tiles - lev) * kKvBN;               // first key of the item
        int Lq = L, Lk = L, qb = 0;                           // query rows [qb, Lq), keys [.., Lk)
        if (R) {
            const i32x4 rg = *reinterpret_cast<const i32x4*>(p.ranges + 4 * wi.seq);
            qb = rg[0]; Lq = min(L, rg[1]); Lk = min(L, rg[3]);
            if (j0 < rg[2] || j0 >= Lk) {                     // the whole key tile is outside the range
                have = wf.next(p.hm, p.cursors, p.items, slot, wi);
                continue;
            }
        }
        const int wkey0 = j0 + 32 * pair;                     // first key of this wave pair
        const int key = wkey0 + l32;
        const bool active = wkey0 < Lk;
        const int qt_first = max(j0, qb) / kKvBM;             // first query tile that sees key j0
        const int n_qt = max((Lq + kKvBM - 1) / kKvBM - qt_first, 0);
        const int n_iter = n_qt * G;
        // rows past the query range read as zeros (as rows past the sequence do)
        const uint32_t q_bytes = (uint32_t)(max(Lq, 1) - 1) * q_stride_b + kRowB;
        const uint32_t stat_bytes = (uint32_t)Lq * 4;

        // stage load of iteration `it` = (query tile it / G, query head it % G of the group): the heads
        // are the inner loop, so that workgroups on neighbouring key tiles of a sequence move through
        // its query tiles at the same pace and find some of each other's Q / dO tiles in L2;
        // every wave issues exactly kDmaPerStage loads, so that a vmcnt wait can tell stages apart
        constexpr int kDmaPerStage = 2 * (16 / kKvWaves) + 1;
        // the loads are issued for it = 0, 1, 2, ... in turn: (tile, head) advance with them instead
        // of being divided out of `it` every time
        int ld_qt = qt_first, ld_h = 0;
        auto dma_stage = [&](int stage) {
            const int h = g * G + ld_h;
            const int qt = ld_qt;
            if (++ld_h == G) { ld_h = 0; ++ld_qt; }
            const int64_t base = (int64_t)row0 * q_stride + (int64_t)h * D;
            const __amdgpu_buffer_rsrc_t rq = make_rsrc(p.sc.q16 + base, q_bytes);
            const __amdgpu_buffer_rsrc_t rdo = make_rsrc(p.sc.do16 + base, q_bytes);
            char* dst = smem + stage * kKvStageBytes + 4 * wave * kRowBytes;
#pragma unroll
            for (int j = 0; j < 16 / kKvWaves; ++j) {
                const uint32_t soff = (uint32_t)qt * tile_bytes + (uint32_t)(j * kKvWaves * 4) * q_stride_b;
                char* d = dst + j * kKvWaves * 4 * kRowBytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rq, (lds_void_b*)d, 16, dma_voff, soff, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rdo, (lds_void_b*)(d + kKvTileBytes), 16, dma_voff, soff, 0, 0);
            }
            // LSE2 and D of the tile's 64 rows: one 256-byte load each, by waves 0 and 1 (the other
            // waves repeat wave 1's load so that all waves count alike); rows past the sequence
            // read as 0, which is harmless because their Q and dO rows are 0 too
            const int which = wave == 0 ? 0 : 1;
            const float* src = (which == 0 ? p.sc.lse2 : p.sc.Dkv) + (int64_t)h * p.T + row0;
            const __amdgpu_buffer_rsrc_t rs = make_rsrc(src, stat_bytes);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_b*)(smem + stage * kKvStageBytes + 2 * kKvTileBytes + which * kKvBM * 4),
                                                     4, (uint32_t)lane * 4, (uint32_t)qt * kKvBM * 4, 0, 0);
        };
        if (n_iter > 0) dma_stage(0);
        if (n_iter > 1) dma_stage(1);

        {   // keys j0 .. j0+127 of K and V of this KV head; rows past the key range read as zeros
            static_assert(kKvBN == 128 && kKvPairs * 2 * kKvPBytes >= kKvBN * kRowBytes, "K/V staging");
            const uint32_t k_bytes = (uint32_t)(min(Lk - j0, kKvBN) - 1) * kv_stride_b + kRowB;
            const int64_t off = (int64_t)(row0 + j0) * kv_stride + (int64_t)g * D;
            dma_rows<kKvWaves>(make_rsrc(p.sc.k16 + off, k_bytes), smem + 2 * kKvStageBytes, [](int j) { return j * kKvTileBytes; },
                               kKvBN / 64, kv_stride_b, wave, dma_voff_kv);
            dma_rows<kKvWaves>(make_rsrc(p.v + off, k_bytes), smem + kKvPOff, [](int j) { return j * kKvTileBytes; },
                               kKvBN / 64, kv_stride_b, wave, dma_voff_kv);
        }
        f32x16 acc[NDB];                                      // dV^T (role A) or dK^T (role B)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
        __syncthreads();                                      // stages 0 and 1 and the K / V rows have landed
        // this wave's register operand of the first product: K rows (role A, fp16 already) or V
        // rows (role B, converted from bf16 here)
        bf16x8 bf[NK];
        {
            u32x4 a[NK];
#pragma unroll
            for (int ks = 0; ks < NK; ++ks) a[ks] = *(lds_u32x4*)(uintptr_t)(fa.row[ks] + kv_stage);
            __builtin_amdgcn_s_waitcnt(0xc07f);               // lgkmcnt(0)
#pragma unroll
            for (int ks = 0; ks < NK; ++ks) {
                asm volatile("" : "+v"(a[ks]));               // the reads stay on this side of the barrier
                if (role_b) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[ks][e] = bf16x2_to_f16x2(a[ks][e]);
                } else {
                    a[ks] ^= sign_flip;
                }
                bf[ks] = as_bf16x8(a[ks]);
            }
        }
        __builtin_amdgcn_s_barrier();                         // stage 2 and the P area may be written now

        // one 32-row block: rows 32*ib.. of the tile in `base`; `parity` selects the P buffer.  The role
        // is a compile-time tag: each role runs its own copy of the tile loop, so that no register
        // has to be reconciled where the roles' paths would join.
        auto block = [&](auto role_tag, int base, int ib, int parity, int qt0) {       // base: LDS offset of the stage
            constexpr bool kB = decltype(role_tag)::value;
            // the role's choice of tile (first product reads Q (A) / dO (B), second product reads
            // dO (A) / Q (B)) is folded into fa.row / fa.col once per kernel
            const int T1 = base, T2 = base;
            const float* stat = reinterpret_cast<const float*>(smem + base + 2 * kKvTileBytes) + (kB ? kKvBM : 0);
            const int ifirst = qt0 + 32 * ib;                 // first query row of the block
            const bool work = active && ifirst + 31 >= wkey0; // some row sees some key of the pair
            f32x16 x;
            uint32_t pk[8];
            constexpr int kCAhead = 4;
            LdsQueue lq{0};
            ColFrag cf[kCAhead];
            if (work) {
                // accumulator slot 4*rq + e holds row 8*rq + 4*half + e of the block: role B's product
                // starts from -D of that row, role A's from zero (its statistic enters after the scale)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    f32x4 i4 = {0.f, 0.f, 0.f, 0.f};
                    if (kB) i4 = *reinterpret_cast<const f32x4*>(stat + 32 * ib + 8 * rq + 4 * half);
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[4 * rq + e] = i4[e];
                }
                // role A's -LSE2 values are requested before the product, so that they are there when
                // the scores are (LDS reads return in order: the first fragment's wait covers them)
                f32x4 l4[4];
                if (!kB) {
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) l4[rq] = *reinterpret_cast<const f32x4*>(stat + 32 * ib + 8 * rq + 4 * half);
                }
                constexpr int kAhead = NK < 6 ? NK : 6;
                bf16x8 f[kAhead];
#pragma unroll
                for (int i = 0; i < kAhead; ++i) f[i] = frag_row(T1, fa, ib, i);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < NK; ++i) {
                    x = mfma32h(f[i % kAhead], bf[i], x);
                    if (i + kAhead < NK) f[i % kAhead] = frag_row(T1, fa, ib, i + kAhead);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (!kB) {
                    if (ifirst < wkey0 + 31) {                // the block straddles the diagonal
                        const int irel = key - ifirst;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (irel > 8 * (r >> 2) + 4 * half + (r & 3)) x[r] = -INFINITY;
                    }
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const f32x4 l4r = l4[rq];                                     // -LSE2
                        f32x4 pv;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            pv[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[4 * rq + e], scale_log2, l4r[e]));
                        // one fp16 rounding of P serves both this wave's dV product and role B
                        pk[2 * rq] = pack_f16(pv[0], pv[1]);
                        pk[2 * rq + 1] = pack_f16(pv[2], pv[3]);
                        const u32x2 hv = {pk[2 * rq], pk[2 * rq + 1]};
                        *reinterpret_cast<u32x2*>(pbuf + parity * kKvPBytes + rq * 512) = hv;
                    }
                }
                // the first fragments of the second product are requested BEFORE the barrier (their
                // tile has been resident since the step began), so that their latency runs under
                // the barrier instead of after it.  LDS operations complete in order: once at most
                // these 2 * kCAhead reads are outstanding, the P stores issued before them are done.
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < kCAhead; ++i) issue_col(lq, cf[i], T2, fa, 2 * ib + i / NDB, i % NDB);
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(0xc07f | ((2 * kCAhead) << 8));
            } else {
                __builtin_amdgcn_s_waitcnt(0xc07f);
            }
            __builtin_amdgcn_s_barrier();
            // Role B is served first on the SIMD the pair shares from here to the end of its dK product:
            // it comes out of the barrier with the longer way to go (the P values have to come back
            // from LDS before it can form dS, while role A's dV operands are in registers), and
            // without the priority its dK MFMAs alternate with A's next score chain, which makes B
            // the late one at the next barrier (A waited 16 % of a block for it, now both wait 5-7 %).
            if (kB) __builtin_amdgcn_s_setprio(3);
            if (work) {
                if (kB) {
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const f16x4 hv = *reinterpret_cast<const f16x4*>(pbuf + parity * kKvPBytes + rq * 512);
                        // written as fused multiply-adds with a zero addend so that the fp16 factor is
                        // converted inside the instruction (v_fma_mix_f32) instead of by one of its own
                        pk[2 * rq] = pack_f16(__builtin_fmaf((float)hv[0], x[4 * rq], 0.f), __builtin_fmaf((float)hv[1], x[4 * rq + 1], 0.f));
                        pk[2 * rq + 1] = pack_f16(__builtin_fmaf((float)hv[2], x[4 * rq + 2], 0.f), __builtin_fmaf((float)hv[3], x[4 * rq + 3], 0.f));
                    }
                }
                // the bookkeeping of the reads issued before the barrier, restated as constants
                lq.issued = 2 * kCAhead;
#pragma unroll
                for (int i = 0; i < kCAhead; ++i) cf[i].seq = 2 * (i + 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 2 * NDB; ++i) {           // i = NDB*b2 + db
                    const int b2 = i / NDB, db = i % NDB;
                    u32x4 bv = {pk[4 * b2], pk[4 * b2 + 1], pk[4 * b2 + 2], pk[4 * b2 + 3]};
                    acc[db] = mfma32h(lds_wait(lq, cf[i % kCAhead]), as_bf16x8(bv), acc[db]);
                    if (i + kCAhead < 2 * NDB) issue_col(lq, cf[i % kCAhead], T2, fa, 2 * ib + (i + kCAhead) / NDB, (i + kCAhead) % NDB);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (kB) __builtin_amdgcn_s_setprio(0);
        };
        int cp_qt = qt_first, cp_h = 0;
        auto step = [&](auto role_tag, auto stage_tag, int it) {
            constexpr int ST = decltype(stage_tag)::value;
            constexpr int ST2 = (ST + 2) % kKvStages;
            constexpr int base = ST * kKvStageBytes;
            const bool more2 = it + 2 < n_iter;
            const int qt0 = cp_qt * kKvBM;                    // the steps advance through (tile, head) like the loads
            if (++cp_h == G) { cp_h = 0; ++cp_qt; }
            block(role_tag, base, 0, 0, qt0);
            // every wave has passed this step's first barrier, hence finished the previous step:
            // the stage that held it may be overwritten now
            if (more2) dma_stage(ST2);
            // the barrier of the second block also opens the next stage: its loads were issued one
            // step ago and precede this step's loads in the (in-order) vmcnt queue
            if (more2) __builtin_amdgcn_s_waitcnt(0x0F70 | (kDmaPerStage & 15) | ((kDmaPerStage >> 4) << 14));
            else __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
            block(role_tag, base, 1, 1, qt0);
        };
        auto tiles = [&](auto role_tag) {
            for (int it = 0; it < n_iter; it += 3) {
                step(role_tag, std::integral_constant<int, 0>{}, it);
                if (it + 1 < n_iter) step(role_tag, std::integral_constant<int, 1>{}, it + 1);
                if (it + 2 < n_iter) step(role_tag, std::integral_constant<int, 2>{}, it + 2);
            }
        };
        if (role_b) tiles(std::true_type{});
        else tiles(std::false_type{});
        __syncthreads();                                      // every wave is done with the ring
        if (active)
            store_rows_via_lds<D>((role_b ? p.dk : p.dv) + (int64_t)(row0 + wkey0) * kv_stride + (int64_t)g * D, kv_stride,
                               Lk - wkey0, acc, (role_b ? p.scale : 1.f) * unscale, o_stage, lane);
        have = wf.next(p.hm, p.cursors, p.items, slot, wi);
    }
    trace_write(p.tr, 1, t_start, n_done);
}

}  // namespace hyd
