// bf16 forward kernel: block-diagonal causal flash-style tile loop on MFMA with fp32 accumulation.
//
// Work item = (sequence, query tile of 256 rows, query head).  A workgroup has 8 waves; wave w
// owns query rows 32w..32w+31 of the tile for the whole item, so the online softmax never crosses
// waves.  K/V tiles of 64 keys travel global -> LDS by direct-to-LDS buffer loads (no staging
// registers, no LDS store instructions) into a ring of three stages shared by the waves: while
// tile t is consumed, tiles t+1 and t+2 are in flight.  One barrier per tile.  The Q rows of an
// item come in the same way and are picked up from LDS as fragments; O leaves through LDS too, so
// that every access to HBM covers whole 256-byte rows.
//
// Orientation.  Scores are computed transposed, S^T[key][q] = K Q^T, so that in the accumulator
// lane map (see mfma32) a lane owns ONE query row (column l%32) and 16 keys per 32-key block:
// the row maximum and row sum are in-lane reductions plus one exchange with the other half of
// the wave, and the softmax statistics are per-lane scalars.  The probabilities then feed
// O^T[d][q] = V^T P^T directly as the B operand (contraction index = key = accumulator row),
// while V^T fragments come out of the row-major V tile with the transposing LDS read.
//
// Reference maximum.  P = exp2(s - m_ref) is exact for ANY per-row reference m_ref as long as it
// neither overflows nor loses the row, so m_ref is only moved (and O, l rescaled) when a tile's
// row maximum exceeds it by more than 8 in the log2 domain; P then stays below 2^8.
//
// Causality.  A wave's 32 rows and the 32-key blocks are aligned, so a block is fully visible,
// fully hidden, or THE diagonal block of the wave (key index in block > row index in block is
// masked).  A wave's diagonal tile is its last, and every tile it computes holds at least one
// visible key for every row, so row maxima are finite.
#pragma once
#include <type_traits>

#include "hyd_sched.h"

namespace hyd {

constexpr int kFwdWaves = 8;
constexpr int kFwdBM = 32 * kFwdWaves, kFwdBN = 64, kFwdThreads = 64 * kFwdWaves;
constexpr int kFwdStages = 3;
constexpr int kFwdTileBytes = kFwdBN * kRowBytes;                 // 16 KB
constexpr int kFwdStageBytes = 2 * kFwdTileBytes;                 // K tile, then V tile
// Q staging: the item's 256 Q rows arrive by direct-to-LDS loads (whole rows per instruction, as
// the K/V tiles do) in four 64-row tiles: two in a region of their own, two in the ring's last
// stage, which no K/V tile needs before the first step.
constexpr int kFwdQxOff = kFwdStages * kFwdStageBytes;
constexpr int kFwdQxBytes = 2 * kFwdTileBytes;
constexpr int kFwdLds = kFwdQxOff + kFwdQxBytes + 64;                 // ring + Q staging + work slot
__device__ __forceinline__ constexpr int fwd_q_stage_off(int j) {
    return j < 2 ? kFwdQxOff + j * kFwdTileBytes : (kFwdStages - 1) * kFwdStageBytes + (j - 2) * kFwdTileBytes;
}
constexpr float kRefSlack = 8.f;                                  // log2 units, see "Reference maximum"

struct FwdParams {
    const uint16_t* q; const uint16_t* k; const uint16_t* v;
    uint16_t* o; float* lse;
    int T, hq, hkv;
    float scale_log2;                 // softmax_scale * log2(e)
    const int* hdr; int* cursors; const int* items;
    HeadMap hm;
    WgTrace tr;
    const int32_t* ranges;            // range variant only: per sequence (q_begin, q_end, kv_begin, kv_end)
    const double* rope_tab;           // NULL, or the rotary frequency table: Q rows are rotated as they are picked up
};

typedef __attribute__((address_space(3))) void lds_void;

// One 64-key tile for the 32 rows of a wave.  There is ONE body for all tiles (separate bodies for
// masked and unmasked tiles make the compiler keep the accumulators twice and copy them at every
// join); only the masking itself sits in a wave-uniform branch.  `diag`: this is the wave's
// diagonal tile (its second 32-key block may be hidden altogether).
// D: head dimension (128 or 64): D/16 contraction steps in the score product, D/32 output blocks.
template <int D>
__device__ __forceinline__ void fwd_tile(int Kt, int Vt, const FragAddr& fa, const bf16x8 (&qf)[D / 16],
                                         f32x16 (&acc_o)[D / 32], float& m_ref, float& l_run, float scale_log2,
                                         int koff, bool diag) {
    constexpr int NK = D / 16, NDB = D / 32;
    // The instruction order below is pinned with scheduling fences: left alone, the compiler sinks
    // every LDS read next to its use and serialises read -> wait -> MFMA.
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
    {
        // fragment i = (contraction step i/2, key block i%2); reads run kAhead fragments ahead
        constexpr int kAhead = 6;
        bf16x8 kf[kAhead];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) kf[i] = frag_row(Kt, fa, i & 1, i >> 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2 * NK; ++i) {
            s[i & 1] = mfma32(kf[i % kAhead], qf[i >> 1], s[i & 1]);
            if (i + kAhead < 2 * NK) kf[i % kAhead] = frag_row(Kt, fa, (i + kAhead) & 1, (i + kAhead) >> 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // the first V fragments are requested now, so that their latency hides behind the softmax
    constexpr int kVAhead = 4;
    LdsQueue lq{0};
    ColFrag vf[kVAhead];
#pragma unroll
    for (int i = 0; i < kVAhead; ++i) issue_col(lq, vf[i], Vt, fa, i / NDB, i % NDB);
    __builtin_amdgcn_sched_barrier(0);
    if (diag) {         // hidden keys score -inf (scale_log2 > 0 always, so exp2 turns them into 0)
        // koff = position of the tile's first key slot of this lane minus the lane's query row.
        // It is formed from the tile index, so that these 32 comparisons stay inside this rarely
        // taken branch (as loop invariants they would be hoisted into 64 scalar registers and
        // spilled at every item).
        const int k0 = koff;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (32 * kb + 8 * (r >> 2) + (r & 3) + k0 > 0) s[kb][r] = -INFINITY;
    }
    // row maximum of the raw scores (a negative softmax scale has been folded into the sign of
    // the Q fragments, so the largest raw score is the largest scaled score)
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    {
        float lo, hi;
        both_halves(mx, lo, hi);
        mx = fmaxf(lo, hi);
    }
    const float cand = mx * scale_log2;
    if (__builtin_expect(__any(cand > m_ref + kRefSlack), 0)) {   // a row left the slack window
        const float m_new = fmaxf(m_ref, cand);
        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[db][r] *= alpha;
        m_ref = m_new;
    }
    // P V: the exponentials of key step b+1 (8 scores) issue under the NDB MFMAs of step b (two
    // scores per MFMA for D = 128, four for D = 64); V fragments are read kVAhead MFMAs ahead.
    float lsum = 0.f;
    auto exp_pair = [&](int j) -> uint32_t {           // scores 2j, 2j+1 of the 32 a lane holds
        const int kb = j >> 3, r = (2 * j) & 15;
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r], scale_log2, -m_ref));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r + 1], scale_log2, -m_ref));
        const uint32_t pair = pack_bf16(p0, p1);
        // row sum of the ROUNDED probabilities (what the P V product actually uses)
        bf16x2 pr;
        __builtin_memcpy(&pr, &pair, 4);
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        lsum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum, false);
        return pair;
    };
    u32x4 pcur, pnxt;
#pragma unroll
    for (int e = 0; e < 4; ++e) pcur[e] = exp_pair(e);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 4 * NDB; ++i) {                 // i = NDB*b + db
        const int b = i / NDB, db = i % NDB;
        acc_o[db] = mfma32(lds_wait(lq, vf[i % kVAhead]), as_bf16x8(pcur), acc_o[db]);
        if (i + kVAhead < 4 * NDB) issue_col(lq, vf[i % kVAhead], Vt, fa, (i + kVAhead) / NDB, (i + kVAhead) % NDB);
        if (b < 3) {
#pragma unroll
            for (int e = 0; e < 4 / NDB; ++e) pnxt[(4 / NDB) * db + e] = exp_pair(4 * (b + 1) + (4 / NDB) * db + e);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (db == NDB - 1) pcur = pnxt;
    }
    l_run += lsum;
}

// R: range variant.  Each sequence has a query range [q_begin, q_end) and a key range
// [kv_begin, kv_end) in local positions, the begins multiples of the query tile: query tiles
// outside the query range are skipped, the tile loop starts at the key range's first tile and
// stops at its end, and a row that sees no key of the range gets O = 0 and LSE = -inf (the
// neutral element of the log-sum-exp merge of partial results).
template <bool R, int D = kHeadDim>
__global__ void __launch_bounds__(kFwdThreads, 1) hyd_fwd_bf16_kernel(FwdParams p) {
    static_assert(D == 128 || D == 64, "head dimension");
    constexpr int kRowB = D * 2;                                      // bytes of a row in global memory
    extern __shared__ __attribute__((aligned(16))) char smem[];
    static_assert(kFwdBM == 256 && kFwdStages == 3, "the Q staging assumes a 256-row tile and a free third stage");
    int* slot = reinterpret_cast<int*>(smem + kFwdQxOff + kFwdQxBytes);
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
    // direct-to-LDS tile load: instruction j of wave w fills tile rows 4*(j*NW + w) .. +3 (1 KB,
    // lane i -> row i/16, chunk position i%16), so lane i fetches the chunk that swz() puts there
    const int dma_row = 4 * wave + (lane >> 4);
    const uint32_t dma_voff = dma_lane_voff<D>(dma_row, lane, kv_stride_b);
    const uint32_t dma_voff_q = dma_lane_voff<D>(dma_row, lane, q_stride_b);
    const uint32_t tile_bytes = kFwdBN * kv_stride_b;                 // one K/V tile in global memory
    // this wave's 32 Q rows inside the staging area, and its private 8 KB of the (free) ring for O
    const int q_stage = ((wave >> 1) < 2 ? kFwdQxOff + (wave >> 1) * kFwdTileBytes
                                         : (kFwdStages - 1) * kFwdStageBytes + ((wave >> 1) - 2) * kFwdTileBytes) +
                        (wave & 1) * 32 * kRowBytes;
    const uint32_t o_stage = (uint32_t)(uintptr_t)(lds_char*)smem + (uint32_t)(wave * 32 * kRowBytes);   // absolute LDS address
    // scale * s = |scale| * (-s): a negative scale flips the sign bits of the Q fragments instead
    // (and a zero scale becomes a denormal-free epsilon, so that -inf * scale stays -inf)
    const float scale_log2 = fmaxf(fabsf(p.scale_log2), 1e-30f);
    const uint32_t sign_flip = p.scale_log2 < 0.f ? 0x80008000u : 0u;

    WorkFetcher wf;
    WorkItem wi;
    bool have = wf.first(p.hm, p.hdr, p.cursors, p.items, slot, wi);
    while (have) {
        ++n_done;
        const int lev = wi.lev, head = wi.head, row0 = wi.row0, L = wi.len;
        const int q0 = (lev - 1) * kFwdBM;
        int Lq = L, kb = 0, kcap = L;                     // query rows [.., Lq), keys [kb, kcap)
        if (R) {
            const i32x4 rg = *reinterpret_cast<const i32x4*>(p.ranges + 4 * wi.seq);
            Lq = min(L, rg[1]); kb = max(rg[2], 0); kcap = min(L, rg[3]);
            if (q0 < rg[0] || q0 >= Lq) {                 // the whole query tile is outside the range
                have = wf.next(p.hm, p.cursors, p.items, slot, wi);
                continue;
            }
        }
        const int kv_end = min(kcap, q0 + kFwdBM);
        const int n_kt = (kv_end + kFwdBN - 1) / kFwdBN;
        const int t_lo = R ? kb / kFwdBN : 0;             // first key tile
        const int g = head / G;
        const int wrow0 = q0 + 32 * wave;                 // first query row of this wave
        const int qrow = wrow0 + l32;
        const bool qvalid = qrow < Lq;
        const bool active = wrow0 < Lq;                   // else the wave only helps with the loads
        if (R && kv_end <= kb) {                          // no key of the range is visible to this tile
            if (qvalid) {
                uint16_t* op = p.o + (int64_t)(row0 + qrow) * q_stride + (int64_t)head * D + 4 * half;
                const u32x2 z = {0u, 0u};
#pragma unroll
                for (int i = 0; i < D / 8; ++i) *reinterpret_cast<u32x2*>(op + 8 * i) = z;
                if (half == 0) p.lse[(int64_t)head * p.T + row0 + qrow] = -INFINITY;
            }
            have = wf.next(p.hm, p.cursors, p.items, slot, wi);
            continue;
        }
        const int td = wrow0 / kFwdBN;                    // this wave's diagonal (= last) tile
        const int koff0 = 4 * half - qrow;                // first key slot of the lane minus its query row, tile 0
        // K/V rows [0, kv_end) of this sequence and KV head; reads past them return zero
        const uint32_t kv_bytes = (uint32_t)(kv_end - 1) * kv_stride_b + kRowB;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc(p.k + (int64_t)row0 * kv_stride + (int64_t)g * D, kv_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc(p.v + (int64_t)row0 * kv_stride + (int64_t)g * D, kv_bytes);
        auto dma_tile = [&](int t, int stage) {
            char* dst = smem + stage * kFwdStageBytes + 4 * wave * kRowBytes;
#pragma unroll
            for (int j = 0; j < 16 / kFwdWaves; ++j) {
                const uint32_t soff = (uint32_t)t * tile_bytes + (uint32_t)(j * kFwdWaves * 4) * kv_stride_b;
                char* d = dst + j * kFwdWaves * 4 * kRowBytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lds_void*)d, 16, dma_voff, soff, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_void*)(d + kFwdTileBytes), 16, dma_voff, soff, 0, 0);
            }
        };
        dma_tile(t_lo, 0);
        if (t_lo + 1 < n_kt) dma_tile(t_lo + 1, 1);

        {   // Q rows q0 .. q0+255 of this head; rows past the query range read as zeros
            const uint32_t q_bytes = (uint32_t)(min(Lq - q0, kFwdBM) - 1) * q_stride_b + kRowB;
            dma_rows<kFwdWaves>(make_rsrc(p.q + (int64_t)(row0 + q0) * q_stride + (int64_t)head * D, q_bytes), smem,
                                [](int j) { return fwd_q_stage_off(j); }, kFwdBM / 64, q_stride_b, wave, dma_voff_q);
        }
        f32x16 acc_o[D / 32];
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
        float m_ref = -INFINITY, l_run = 0.f;
        __syncthreads();                                  // the first tiles and the Q rows have landed
        bf16x8 qf[D / 16];
        {
            u32x4 qv[D / 16];
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) qv[ks] = *(lds_u32x4*)(uintptr_t)(fa.row[ks] + (uint32_t)q_stage);
            __builtin_amdgcn_s_waitcnt(0xc07f);           // lgkmcnt(0)
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                asm volatile("" : "+v"(qv[ks]));          // the reads stay on this side of the barrier
            }
            if (p.rope_tab) rope_row_frags<D, false>(qv, p.rope_tab, qrow, half);      // position = local row: reset per sequence
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) qf[ks] = as_bf16x8(qv[ks] ^ sign_flip);
        }
        __builtin_amdgcn_s_barrier();                     // the staged Q may be overwritten (tile t_lo+2 goes there)

        // one tile on ring stage ST (compile-time, so that fragment reads are base+immediate)
        auto step = [&](auto stage_tag, int t) {
            constexpr int ST = decltype(stage_tag)::value;
            constexpr int Kt = ST * kFwdStageBytes, Vt = Kt + kFwdTileBytes;      // LDS offsets of the tiles
            // the loads run two tiles ahead: tile t+1 was requested one step ago and precedes this
            // step's loads in the (in-order) vmcnt queue
            constexpr int ST2 = (ST + 2) % kFwdStages;
            constexpr int kDmaPerTile = 2 * (16 / kFwdWaves);
            const bool more2 = t + 2 < n_kt;
            if (more2) dma_tile(t + 2, ST2);
            if (active && t <= td)
                fwd_tile<D>(Kt, Vt, fa, qf, acc_o, m_ref, l_run, scale_log2, t * kFwdBN + koff0, t == td);
            if (more2) __builtin_amdgcn_s_waitcnt(0x0070 | (kDmaPerTile & 15));     // vmcnt(kDmaPerTile), lgkmcnt(0)
            else __builtin_amdgcn_s_waitcnt(0x0070);                                // vmcnt(0), lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
        };
        for (int t = t_lo; t < n_kt; t += 3) {
            step(std::integral_constant<int, 0>{}, t);
            if (t + 1 < n_kt) step(std::integral_constant<int, 1>{}, t + 1);
            if (t + 2 < n_kt) step(std::integral_constant<int, 2>{}, t + 2);
        }
        // epilogue: normalise, write O (bf16) and LSE (natural log)
        float l_lo, l_hi;
        both_halves(l_run, l_lo, l_hi);
        const float l_tot = l_lo + l_hi;
        // range variant: a row below the key range has l = 0, m = -inf: O = 0, LSE = -inf
        const float inv = (R && !(l_tot > 0.f)) ? 0.f : 1.f / l_tot;
        if (active) {
            // O leaves through this wave's 8 KB of the ring (free now): whole rows per store
            store_rows_via_lds<D>(p.o + (int64_t)(row0 + wrow0) * q_stride + (int64_t)head * D, q_stride, Lq - wrow0,
                               acc_o, inv, o_stage, lane);
            if (qvalid && half == 0)
                p.lse[(int64_t)head * p.T + row0 + qrow] =
                    (m_ref + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
        }
        have = wf.next(p.hm, p.cursors, p.items, slot, wi);
    }
    trace_write(p.tr, 0, t_start, n_done);
}

}  // namespace hyd
