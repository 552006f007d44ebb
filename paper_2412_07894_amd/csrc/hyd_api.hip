// Host side of the C ABI declared in include/hyd_attn.h: argument validation (before any HIP
// call), workspace layout, launch configuration and the benchmark hooks.
#include "../../include/hyd_attn.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "hyd_bwd_bf16.h"
#include "hyd_fp32.h"
#include "hyd_fwd_bf16.h"
#include "hyd_merge.h"
#include "hyd_rope.h"

namespace {

using namespace hyd;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Workspace: one or two schedules (the backward has one per tile size when its two kernels use
// different tiles), then the backward's row statistics ([Hq][T] floats; the fp32 path uses the
// first one only) and, for bf16, the fp16 copies of Q, dO and K that its tile loops stream.
constexpr int kBwdStatVecs = 4;
constexpr int kHdrAbsmax = 40;            // header word of the dK/dV schedule that holds max |dO| (see BwdScratch)
struct SchedLayout { size_t hdr, lev, order, items; int n_lev, max_items; };
struct WsLayout {
    SchedLayout sched[2];
    int n_sched;
    size_t stat[kBwdStatVecs], q16, do16, k16, rope_tab, total;
};
constexpr int kRopeTabEntries = 64;       // head_dim / 2 at most

size_t sched_layout(SchedLayout& v, size_t at, int T, int nseq, int tile) {
    v.n_lev = (T + tile - 1) / tile;
    if (v.n_lev < 1) v.n_lev = 1;
    v.max_items = T / tile + nseq + 1;
    v.hdr = at;   at += align_up(sizeof(int) * kHdrInts);
    v.lev = at;   at += align_up(sizeof(int) * 3 * (size_t)(v.n_lev + 2));
    v.order = at; at += align_up(sizeof(int) * (size_t)(nseq > 0 ? nseq : 1));
    v.items = at; at += align_up(sizeof(int) * 4 * (size_t)v.max_items);
    return at;
}

WsLayout ws_layout(int T, int nseq, int tile0, int tile1, int hq, int hkv, int head_dim, hyd_dtype dt, bool bwd) {
    WsLayout w;
    size_t at = sched_layout(w.sched[0], 0, T, nseq, tile0);
    w.n_sched = tile1 != tile0 ? 2 : 1;
    if (w.n_sched == 2) at = sched_layout(w.sched[1], at, T, nseq, tile1);
    else w.sched[1] = w.sched[0];
    const int n_stat = !bwd ? 0 : (dt == HYD_BF16 ? kBwdStatVecs : 1);
    for (int i = 0; i < kBwdStatVecs; ++i) {
        w.stat[i] = at;
        if (i < n_stat) at += align_up(sizeof(float) * (size_t)T * (size_t)hq);
    }
    const bool copies = bwd && dt == HYD_BF16;
    w.q16 = at;  if (copies) at += align_up(2 * (size_t)T * (size_t)hq * (size_t)head_dim);
    w.do16 = at; if (copies) at += align_up(2 * (size_t)T * (size_t)hq * (size_t)head_dim);
    w.k16 = at;  if (copies) at += align_up(2 * (size_t)T * (size_t)hkv * (size_t)head_dim);
    w.rope_tab = at; at += align_up(sizeof(double) * kRopeTabEntries);       // rotary frequency table (the *_rope calls)
    w.total = at;
    return w;
}

// rows per work item of the forward and of the backward kernels
int tile_fwd(hyd_dtype dt) { return dt == HYD_BF16 ? kFwdBM : kF32Tile; }
int tile_dq(hyd_dtype dt) { return dt == HYD_BF16 ? kDqBM : kF32Tile; }
int tile_kv(hyd_dtype dt) { return dt == HYD_BF16 ? kKvBN : kF32Tile; }


bool head_dim_ok(hyd_dtype dt, int d) { (void)dt; return d == 64 || d == 128; }

// Spread of (item, head) pairs over the 8 queues: whole KV groups per queue when the KV heads
// divide over the queues, else single heads, else items striped with all heads in every queue.
HeadMap head_map_q(int hq, int hkv) {
    HeadMap hm;
    hm.heads = hq;
    if (hkv % kQueues == 0) { hm.striped = 0; hm.hpq = hq / kQueues; hm.group = hq / hkv; }
    else if (hq % kQueues == 0) { hm.striped = 0; hm.hpq = hq / kQueues; hm.group = 1; }
    else { hm.striped = 1; hm.hpq = hq; hm.group = 1; }
    return hm;
}
HeadMap head_map_kv(int hkv) {
    HeadMap hm;
    hm.heads = hkv;
    if (hkv % kQueues == 0) { hm.striped = 0; hm.hpq = hkv / kQueues; hm.group = 1; }
    else { hm.striped = 1; hm.hpq = hkv; hm.group = 1; }
    return hm;
}

hyd_status validate_common(const int32_t* cu, int num_seqs, const int32_t* cu_host, int T,
                           int max_seqlen, int hq, int hkv, int head_dim, hyd_dtype dt,
                           const void* ws, size_t ws_bytes, bool bwd) {
    if (dt != HYD_BF16 && dt != HYD_FP32) return HYD_ERR_DTYPE;
    if (T < 0 || num_seqs < 0 || max_seqlen < 0) return HYD_ERR_SHAPE;
    if (num_seqs == 0 && T != 0) return HYD_ERR_SHAPE;
    if (hq <= 0 || hkv <= 0 || hq % hkv != 0) return HYD_ERR_HEADS;
    if (!head_dim_ok(dt, head_dim)) return HYD_ERR_HEADDIM;
    if (T == 0 || num_seqs == 0) return HYD_OK;
    if (!cu) return HYD_ERR_NULL;
    if (max_seqlen > T || max_seqlen < 1) return HYD_ERR_SHAPE;
    // a sequence must fit the 32-bit range of a buffer resource based at its first row
    if ((unsigned long long)max_seqlen * (unsigned long long)hq * (unsigned long long)head_dim *
            (dt == HYD_BF16 ? 2ull : 4ull) >= (dt == HYD_BF16 && head_dim == 64 ? (1ull << 31) : (1ull << 32)))
        return HYD_ERR_SHAPE;
    if (cu_host) {
        if (cu_host[0] != 0 || cu_host[num_seqs] != T) return HYD_ERR_SEQLENS;
        int longest = 0;
        for (int s = 0; s < num_seqs; ++s) {
            const int L = cu_host[s + 1] - cu_host[s];
            if (L < 0) return HYD_ERR_SEQLENS;
            if (L > longest) longest = L;
        }
        if (longest > max_seqlen) return HYD_ERR_SHAPE;
    }
    const size_t need = hyd_varlen_attn_workspace_bytes(T, num_seqs, hq, hkv, head_dim, dt, bwd ? 1 : 0);
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < need) return HYD_ERR_WORKSPACE;
    return HYD_OK;
}

// Range variants: begins must fall on the coarsest tile boundary of the three kernels, ends
// either there or at / past the end of the sequence (then the sequence's length caps them).
static_assert(HYD_RANGE_ALIGN % kFwdBM == 0 && HYD_RANGE_ALIGN % kDqBM == 0 && HYD_RANGE_ALIGN % kKvBN == 0 &&
              HYD_RANGE_ALIGN % kFwdBN == 0 && HYD_RANGE_ALIGN % kDqBN == 0 && HYD_RANGE_ALIGN % kKvBM == 0,
              "range granule must be a multiple of every tile size");

hyd_status validate_ranges(const int32_t* ranges, const int32_t* ranges_host, const int32_t* cu_host,
                           int num_seqs, int max_seqlen, hyd_dtype dt) {
    if (dt != HYD_BF16) return HYD_ERR_DTYPE;
    if (num_seqs == 0) return HYD_OK;
    if (!ranges) return HYD_ERR_NULL;
    if (!ranges_host) return HYD_OK;
    for (int s = 0; s < num_seqs; ++s) {
        const int32_t* r = ranges_host + 4 * s;
        const int L = cu_host ? cu_host[s + 1] - cu_host[s] : max_seqlen;
        for (int e = 0; e < 2; ++e) {
            const int b = r[2 * e], en = r[2 * e + 1];
            if (b < 0 || b % HYD_RANGE_ALIGN != 0 || en < b) return HYD_ERR_RANGE;
            if (en % HYD_RANGE_ALIGN != 0 && en < L) return HYD_ERR_RANGE;
        }
    }
    return HYD_OK;
}

// ---- library-owned scratch of the entry point that allocates nothing ---------------------------
// Holds the forward's workspace (one schedule) for callers that cannot provide one.  Every GPU the
// library runs on keeps its own copy of this array until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the address kernels and memory calls use
// is DeviceInfo::scratch, looked up once per device.
constexpr size_t kScratchBytes = 2u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// ---- per-device state -------------------------------------------------------------------------
struct DeviceInfo {
    bool ready = false, ok = false;
    int cus = 0;
    int occ_fwd = 1, occ_dq = 1, occ_kv = 1;
    void* scratch = nullptr;          // this device's copy of the array above
};
DeviceInfo g_dev[64];
std::mutex g_dev_mutex;       // first use of a device from several host threads at once

template <typename K>
bool prep_kernel(K kernel, int threads, int lds, int* occ) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
        return false;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, lds) != hipSuccess) return false;
    if (occ) *occ = n < 1 ? 1 : n;
    return true;
}

hyd_status device_info(DeviceInfo** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HYD_ERR_LAUNCH;
    if (dev < 0 || dev >= 64) return HYD_ERR_LAUNCH;
    DeviceInfo& d = g_dev[dev];
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (!d.ready) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return HYD_ERR_LAUNCH;
        d.ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        d.cus = prop.multiProcessorCount;
        if (d.ok) {
            if (!prep_kernel(hyd_fwd_bf16_kernel<false>, kFwdThreads, kFwdLds, &d.occ_fwd) ||
                !prep_kernel(hyd_fwd_bf16_kernel<false, 64>, kFwdThreads, kFwdLds, nullptr) ||
                !prep_kernel(hyd_fwd_bf16_kernel<true, 64>, kFwdThreads, kFwdLds, nullptr) ||
                !prep_kernel(hyd_bwd_dq_bf16_kernel<false>, kDqThreads, kDqLds, &d.occ_dq) ||
                !prep_kernel(hyd_bwd_dkdv_bf16_kernel<false>, kKvThreads, kKvLds, &d.occ_kv) ||
                !prep_kernel(hyd_fwd_bf16_kernel<true>, kFwdThreads, kFwdLds, nullptr) ||
                !prep_kernel(hyd_bwd_dq_bf16_kernel<true>, kDqThreads, kDqLds, nullptr) ||
                !prep_kernel(hyd_bwd_dkdv_bf16_kernel<true>, kKvThreads, kKvLds, nullptr) ||
                !prep_kernel(hyd_bwd_dq_bf16_kernel<false, 64>, kDqThreads, kDqLds, nullptr) ||
                !prep_kernel(hyd_bwd_dkdv_bf16_kernel<false, 64>, kKvThreads, kKvLds, nullptr) ||
                !prep_kernel(hyd_bwd_dq_bf16_kernel<true, 64>, kDqThreads, kDqLds, nullptr) ||
                !prep_kernel(hyd_bwd_dkdv_bf16_kernel<true, 64>, kKvThreads, kKvLds, nullptr) ||
                !prep_kernel(hyd_bwd_dkdv_fp32_kernel<64>, kF32Tile, f32_dkdv_lds<64>(), nullptr) ||
                !prep_kernel(hyd_bwd_dkdv_fp32_kernel<128>, kF32Tile, f32_dkdv_lds<128>(), nullptr))
                return HYD_ERR_LAUNCH;
            void* sp = nullptr;
            if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp) return HYD_ERR_LAUNCH;
            d.scratch = sp;
        }
        d.ready = true;
    }
    if (!d.ok) return HYD_ERR_ARCH;
    *out = &d;
    return HYD_OK;
}

// ---- benchmark hooks --------------------------------------------------------------------------
struct TimedKernel { const char* name; hipEvent_t e0, e1; };
thread_local bool t_timing = false;
thread_local std::vector<TimedKernel> t_timed;
thread_local WgTrace t_trace = {nullptr, 0};

void timed_clear() {
    for (auto& t : t_timed) { (void)hipEventDestroy(t.e0); (void)hipEventDestroy(t.e1); }
    t_timed.clear();
}

constexpr size_t kMaxTimed = 8192;      // launches recorded between two reads of the list

struct KernelTimer {       // brackets one launch with events when timing is on
    hipStream_t st; bool on; TimedKernel tk;
    KernelTimer(const char* name, hipStream_t s) : st(s), on(t_timing && t_timed.size() < kMaxTimed) {
        tk.name = name;
        if (on) {
            on = hipEventCreate(&tk.e0) == hipSuccess && hipEventCreate(&tk.e1) == hipSuccess;
            if (on) (void)hipEventRecord(tk.e0, st);
        }
    }
    ~KernelTimer() {
        if (on) { (void)hipEventRecord(tk.e1, st); t_timed.push_back(tk); }
    }
};

// View of schedule `which`; its level count is bounded by the caller's max_seqlen.
SchedView make_view(char* ws, const SchedLayout& v, int tile, int max_seqlen) {
    SchedView sv;
    sv.hdr = reinterpret_cast<int*>(ws + v.hdr);
    sv.lev = reinterpret_cast<int*>(ws + v.lev);
    sv.order = reinterpret_cast<int*>(ws + v.order);
    sv.items = reinterpret_cast<int*>(ws + v.items);
    const int by_len = (max_seqlen + tile - 1) / tile;
    sv.n_lev = by_len < v.n_lev ? (by_len < 1 ? 1 : by_len) : v.n_lev;
    sv.max_items = v.max_items;
    return sv;
}

int persistent_grid(const DeviceInfo& d, int occ, long long work_upper_bound) {
    long long g = (long long)d.cus * occ;
    if (g > work_upper_bound) g = work_upper_bound;
    return g < 1 ? 1 : (int)g;
}

}  // namespace

extern "C" {

const char* hyd_status_string(hyd_status st) {
    switch (st) {
        case HYD_OK: return "HYD_OK";
        case HYD_ERR_NULL: return "HYD_ERR_NULL: a required pointer is NULL";
        case HYD_ERR_SHAPE: return "HYD_ERR_SHAPE: negative size or max_seqlen out of range";
        case HYD_ERR_DTYPE: return "HYD_ERR_DTYPE: unknown dtype";
        case HYD_ERR_HEADS: return "HYD_ERR_HEADS: hq and hkv must be positive with hq % hkv == 0";
        case HYD_ERR_HEADDIM: return "HYD_ERR_HEADDIM: head_dim must be 64 or 128";
        case HYD_ERR_SEQLENS: return "HYD_ERR_SEQLENS: cu_seqlens must start at 0, end at T and not decrease";
        case HYD_ERR_WORKSPACE: return "HYD_ERR_WORKSPACE: workspace NULL, misaligned or too small";
        case HYD_ERR_ARCH: return "HYD_ERR_ARCH: device is not gfx950";
        case HYD_ERR_LAUNCH: return "HYD_ERR_LAUNCH: HIP launch or query failed";
        case HYD_ERR_INFEASIBLE: return "HYD_ERR_INFEASIBLE: the planning constraints admit no solution";
        case HYD_ERR_RANGE: return "HYD_ERR_RANGE: a range begin is not a multiple of HYD_RANGE_ALIGN, or an end is neither that nor past the sequence";
    }
    return "unknown hyd_status";
}

size_t hyd_varlen_attn_workspace_bytes(int total_tokens, int num_seqs, int hq, int hkv, int head_dim,
                                       hyd_dtype dt, int is_bwd) {
    if (total_tokens < 0 || num_seqs < 0 || hq <= 0 || hkv <= 0 || hq % hkv != 0) return 0;
    if ((dt != HYD_BF16 && dt != HYD_FP32) || !head_dim_ok(dt, head_dim)) return 0;
    return (is_bwd ? ws_layout(total_tokens, num_seqs, tile_kv(dt), tile_dq(dt), hq, hkv, head_dim, dt, true)
                   : ws_layout(total_tokens, num_seqs, tile_fwd(dt), tile_fwd(dt), hq, hkv, head_dim, dt, false)).total;
}

}  // extern "C"

namespace {

// forward of the plain entry point (ranges == NULL) and of the range variant
// rope_base: 0 = no rotation, else the base of the rotary embedding applied to Q inside the kernels
hyd_status fwd_impl(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                    int num_seqs, const int32_t* cu_seqlens_host, const int32_t* ranges,
                    const int32_t* ranges_host, bool ranged, int total_tokens,
                    int max_seqlen, int hq, int hkv, int head_dim, float softmax_scale,
                    hyd_dtype dt, void* o, float* lse, void* workspace,
                    size_t workspace_bytes, void* hip_stream, float rope_base = 0.f) {
    if (rope_base != 0.f && (dt != HYD_BF16 || !(rope_base > 1.f))) return dt != HYD_BF16 ? HYD_ERR_DTYPE : HYD_ERR_SHAPE;
    const hyd_status vs = validate_common(cu_seqlens, num_seqs, cu_seqlens_host, total_tokens, max_seqlen,
                                          hq, hkv, head_dim, dt, workspace, workspace_bytes, false);
    if (vs != HYD_OK) return vs;
    if (ranged) {
        const hyd_status rs = validate_ranges(ranges, ranges_host, cu_seqlens_host, num_seqs, max_seqlen, dt);
        if (rs != HYD_OK) return rs;
    }
    if (total_tokens == 0 || num_seqs == 0) return HYD_OK;
    if (!q || !k || !v || !o || !lse) return HYD_ERR_NULL;

    DeviceInfo* dev = nullptr;
    const hyd_status ds = device_info(&dev);
    if (ds != HYD_OK) return ds;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    const int tile = tile_fwd(dt);
    const WsLayout w = ws_layout(total_tokens, num_seqs, tile, tile, hq, hkv, head_dim, dt, false);
    const SchedView sv = make_view(static_cast<char*>(workspace), w.sched[0], tile, max_seqlen);
    double* rope_tab = rope_base != 0.f ? reinterpret_cast<double*>(static_cast<char*>(workspace) + w.rope_tab) : nullptr;
    {
        KernelTimer kt("schedule_prelude", st);
        hipLaunchKernelGGL(hyd_schedule_prelude, dim3(1), dim3(kPreludeThreads), 0, st, cu_seqlens, num_seqs, total_tokens, tile, sv, tile, sv,
                           rope_tab, head_dim / 2, rope_base != 0.f ? log2((double)rope_base) : 0.0);
    }
    const HeadMap hm = head_map_q(hq, hkv);
    const long long work = (long long)sv.max_items * hq;
    if (dt == HYD_BF16) {
        FwdParams p;
        p.q = static_cast<const uint16_t*>(q); p.k = static_cast<const uint16_t*>(k);
        p.v = static_cast<const uint16_t*>(v); p.o = static_cast<uint16_t*>(o); p.lse = lse;
        p.T = total_tokens; p.hq = hq; p.hkv = hkv;
        p.scale_log2 = softmax_scale * kLog2e;
        p.hdr = sv.hdr; p.cursors = sv.hdr + kHdrCursor; p.items = sv.items; p.hm = hm; p.tr = t_trace;
        p.ranges = ranged ? ranges : nullptr;
        p.rope_tab = rope_tab;
        const dim3 grid(persistent_grid(*dev, dev->occ_fwd, work));
        KernelTimer kt(ranged ? "fwd_range_bf16" : "fwd_bf16", st);
        if (head_dim == 64) {
            if (ranged) hipLaunchKernelGGL((hyd_fwd_bf16_kernel<true, 64>), grid, dim3(kFwdThreads), kFwdLds, st, p);
            else hipLaunchKernelGGL((hyd_fwd_bf16_kernel<false, 64>), grid, dim3(kFwdThreads), kFwdLds, st, p);
        } else if (ranged) hipLaunchKernelGGL(hyd_fwd_bf16_kernel<true>, grid, dim3(kFwdThreads), kFwdLds, st, p);
        else hipLaunchKernelGGL(hyd_fwd_bf16_kernel<false>, grid, dim3(kFwdThreads), kFwdLds, st, p);
    } else {
        F32Params p;
        memset(&p, 0, sizeof(p));
        p.q = static_cast<const float*>(q); p.k = static_cast<const float*>(k);
        p.v = static_cast<const float*>(v); p.o_out = static_cast<float*>(o); p.lse_out = lse;
        p.T = total_tokens; p.hq = hq; p.hkv = hkv; p.scale = softmax_scale;
        p.hdr = sv.hdr; p.cursors = sv.hdr + kHdrCursor; p.items = sv.items; p.hm = hm; p.tr = t_trace;
        const int grid = persistent_grid(*dev, 8, work);
        KernelTimer kt("fwd_fp32", st);
        if (head_dim == 64) hipLaunchKernelGGL(hyd_fwd_fp32_kernel<64>, dim3(grid), dim3(kF32Tile), 0, st, p);
        else hipLaunchKernelGGL(hyd_fwd_fp32_kernel<128>, dim3(grid), dim3(kF32Tile), 0, st, p);
    }
    return hipGetLastError() == hipSuccess ? HYD_OK : HYD_ERR_LAUNCH;
}

// backward of the plain entry point (ranges == NULL) and of the range variant
hyd_status bwd_impl(const void* q, const void* k, const void* v, const void* o, const float* lse,
                    const void* d_o, const int32_t* cu_seqlens, int num_seqs,
                    const int32_t* cu_seqlens_host, const int32_t* ranges, const int32_t* ranges_host,
                    bool ranged, int total_tokens, int max_seqlen, int hq,
                    int hkv, int head_dim, float softmax_scale, hyd_dtype dt, void* dq, void* dk,
                    void* dv, void* workspace, size_t workspace_bytes, void* hip_stream, float rope_base = 0.f) {
    if (rope_base != 0.f && (dt != HYD_BF16 || !(rope_base > 1.f))) return dt != HYD_BF16 ? HYD_ERR_DTYPE : HYD_ERR_SHAPE;
    const hyd_status vs = validate_common(cu_seqlens, num_seqs, cu_seqlens_host, total_tokens, max_seqlen,
                                          hq, hkv, head_dim, dt, workspace, workspace_bytes, true);
    if (vs != HYD_OK) return vs;
    if (ranged) {
        const hyd_status rs = validate_ranges(ranges, ranges_host, cu_seqlens_host, num_seqs, max_seqlen, dt);
        if (rs != HYD_OK) return rs;
    }
    if (total_tokens == 0 || num_seqs == 0) return HYD_OK;
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv) return HYD_ERR_NULL;

    DeviceInfo* dev = nullptr;
    const hyd_status ds = device_info(&dev);
    if (ds != HYD_OK) return ds;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    const WsLayout w = ws_layout(total_tokens, num_seqs, tile_kv(dt), tile_dq(dt), hq, hkv, head_dim, dt, true);
    char* ws = static_cast<char*>(workspace);
    const SchedView sv_kv = make_view(ws, w.sched[0], tile_kv(dt), max_seqlen);
    const SchedView sv_q = make_view(ws, w.sched[1], tile_dq(dt), max_seqlen);
    float* Dvec = reinterpret_cast<float*>(ws + w.stat[0]);
    double* rope_tab = rope_base != 0.f ? reinterpret_cast<double*>(ws + w.rope_tab) : nullptr;
    // one launch builds the item list of the dK/dV kernel and, if the dQ kernel uses another tile
    // size, the dQ kernel's too (one workgroup each)
    {
        KernelTimer kt("schedule_prelude", st);
        hipLaunchKernelGGL(hyd_schedule_prelude, dim3(w.n_sched), dim3(kPreludeThreads), 0, st, cu_seqlens, num_seqs, total_tokens,
                           tile_kv(dt), sv_kv, tile_dq(dt), sv_q, rope_tab, head_dim / 2, rope_base != 0.f ? log2((double)rope_base) : 0.0);
    }
    const long long n_rows = (long long)total_tokens * hq;
    const long long work_q = (long long)sv_q.max_items * hq, work_kv = (long long)sv_kv.max_items * hkv;
    if (dt == HYD_BF16) {
        BwdScratch sc;
        sc.Dq = Dvec;
        sc.kqmul = reinterpret_cast<float*>(ws + w.stat[1]);
        sc.lse2 = reinterpret_cast<float*>(ws + w.stat[2]);
        sc.Dkv = reinterpret_cast<float*>(ws + w.stat[3]);
        sc.absmax = reinterpret_cast<uint32_t*>(sv_kv.hdr + kHdrAbsmax);      // the prelude has cleared the header
        sc.q16 = reinterpret_cast<uint16_t*>(ws + w.q16);
        sc.do16 = reinterpret_cast<uint16_t*>(ws + w.do16);
        sc.k16 = reinterpret_cast<uint16_t*>(ws + w.k16);
        {
            KernelTimer kt("bwd_rowstats_bf16", st);
            const int stat_tok = rowstats_tokens(hq);
            const dim3 rgrid((unsigned)((total_tokens + stat_tok - 1) / stat_tok));
            if (head_dim == 64)
                hipLaunchKernelGGL(hyd_bwd_rowstats_bf16_kernel<64>, rgrid, dim3(256), rowstats_lds(hq), st, static_cast<const uint16_t*>(o),
                                   static_cast<const uint16_t*>(d_o), lse, static_cast<const uint16_t*>(k), sc, total_tokens, hq, hkv, stat_tok);
            else
                hipLaunchKernelGGL(hyd_bwd_rowstats_bf16_kernel<kHeadDim>, rgrid, dim3(256), rowstats_lds(hq), st, static_cast<const uint16_t*>(o),
                                   static_cast<const uint16_t*>(d_o), lse, static_cast<const uint16_t*>(k), sc, total_tokens, hq, hkv, stat_tok);
        }
        BwdParams p;
        p.q = static_cast<const uint16_t*>(q); p.v = static_cast<const uint16_t*>(v); p.d_o = static_cast<const uint16_t*>(d_o);
        p.sc = sc;
        p.dq = static_cast<uint16_t*>(dq); p.dk = static_cast<uint16_t*>(dk); p.dv = static_cast<uint16_t*>(dv);
        p.T = total_tokens; p.hq = hq; p.hkv = hkv;
        p.scale = softmax_scale; p.scale_log2 = softmax_scale * kLog2e;
        p.tr = t_trace;
        p.ranges = ranged ? ranges : nullptr;
        p.rope_tab = rope_tab;
        // dQ first: it also writes the fp16 copies of Q and dO that dK/dV streams
        {
            p.hdr = sv_q.hdr; p.items = sv_q.items;
            p.cursors = sv_q.hdr + kHdrCursor + 2 * kQueues; p.hm = head_map_q(hq, hkv);
            const dim3 grid(persistent_grid(*dev, dev->occ_dq, work_q));
            KernelTimer kt(ranged ? "bwd_dq_range_bf16" : "bwd_dq_bf16", st);
            if (head_dim == 64) {
                if (ranged) hipLaunchKernelGGL((hyd_bwd_dq_bf16_kernel<true, 64>), grid, dim3(kDqThreads), kDqLds, st, p);
                else hipLaunchKernelGGL((hyd_bwd_dq_bf16_kernel<false, 64>), grid, dim3(kDqThreads), kDqLds, st, p);
            } else if (ranged) hipLaunchKernelGGL(hyd_bwd_dq_bf16_kernel<true>, grid, dim3(kDqThreads), kDqLds, st, p);
            else hipLaunchKernelGGL(hyd_bwd_dq_bf16_kernel<false>, grid, dim3(kDqThreads), kDqLds, st, p);
        }
        {
            p.hdr = sv_kv.hdr; p.items = sv_kv.items;
            p.cursors = sv_kv.hdr + kHdrCursor + kQueues; p.hm = head_map_kv(hkv);
            const dim3 grid(persistent_grid(*dev, dev->occ_kv, work_kv));
            KernelTimer kt(ranged ? "bwd_dkdv_range_bf16" : "bwd_dkdv_bf16", st);
            if (head_dim == 64) {
                if (ranged) hipLaunchKernelGGL((hyd_bwd_dkdv_bf16_kernel<true, 64>), grid, dim3(kKvThreads), kKvLds, st, p);
                else hipLaunchKernelGGL((hyd_bwd_dkdv_bf16_kernel<false, 64>), grid, dim3(kKvThreads), kKvLds, st, p);
            } else if (ranged) hipLaunchKernelGGL(hyd_bwd_dkdv_bf16_kernel<true>, grid, dim3(kKvThreads), kKvLds, st, p);
            else hipLaunchKernelGGL(hyd_bwd_dkdv_bf16_kernel<false>, grid, dim3(kKvThreads), kKvLds, st, p);
        }
    } else {
        F32Params p;
        memset(&p, 0, sizeof(p));
        p.q = static_cast<const float*>(q); p.k = static_cast<const float*>(k);
        p.v = static_cast<const float*>(v); p.o = static_cast<const float*>(o);
        p.d_o = static_cast<const float*>(d_o); p.lse_in = lse; p.D = Dvec;
        p.dq = static_cast<float*>(dq); p.dk = static_cast<float*>(dk); p.dv = static_cast<float*>(dv);
        p.T = total_tokens; p.hq = hq; p.hkv = hkv; p.scale = softmax_scale;
        p.tr = t_trace;
        const unsigned rd_grid = (unsigned)((n_rows + 255) / 256);
        const int grid_q = persistent_grid(*dev, 8, work_q), grid_kv = persistent_grid(*dev, 2, work_kv);
        if (head_dim == 64) {
            { KernelTimer kt("bwd_rowdot_fp32", st);
              hipLaunchKernelGGL(hyd_bwd_rowdot_fp32_kernel<64>, dim3(rd_grid), dim3(256), 0, st, p.o, p.d_o, Dvec, total_tokens, hq); }
            p.hdr = sv_kv.hdr; p.items = sv_kv.items; p.cursors = sv_kv.hdr + kHdrCursor + kQueues; p.hm = head_map_kv(hkv);
            { KernelTimer kt("bwd_dkdv_fp32", st);
              hipLaunchKernelGGL(hyd_bwd_dkdv_fp32_kernel<64>, dim3(grid_kv), dim3(kF32Tile), f32_dkdv_lds<64>(), st, p); }
            p.hdr = sv_q.hdr; p.items = sv_q.items; p.cursors = sv_q.hdr + kHdrCursor + 2 * kQueues; p.hm = head_map_q(hq, hkv);
            { KernelTimer kt("bwd_dq_fp32", st);
              hipLaunchKernelGGL(hyd_bwd_dq_fp32_kernel<64>, dim3(grid_q), dim3(kF32Tile), 0, st, p); }
        } else {
            { KernelTimer kt("bwd_rowdot_fp32", st);
              hipLaunchKernelGGL(hyd_bwd_rowdot_fp32_kernel<128>, dim3(rd_grid), dim3(256), 0, st, p.o, p.d_o, Dvec, total_tokens, hq); }
            p.hdr = sv_kv.hdr; p.items = sv_kv.items; p.cursors = sv_kv.hdr + kHdrCursor + kQueues; p.hm = head_map_kv(hkv);
            { KernelTimer kt("bwd_dkdv_fp32", st);
              hipLaunchKernelGGL(hyd_bwd_dkdv_fp32_kernel<128>, dim3(grid_kv), dim3(kF32Tile), f32_dkdv_lds<128>(), st, p); }
            p.hdr = sv_q.hdr; p.items = sv_q.items; p.cursors = sv_q.hdr + kHdrCursor + 2 * kQueues; p.hm = head_map_q(hq, hkv);
            { KernelTimer kt("bwd_dq_fp32", st);
              hipLaunchKernelGGL(hyd_bwd_dq_fp32_kernel<128>, dim3(grid_q), dim3(kF32Tile), 0, st, p); }
        }
    }
    return hipGetLastError() == hipSuccess ? HYD_OK : HYD_ERR_LAUNCH;
}

}  // namespace

extern "C" {

hyd_status hyd_varlen_attn_fwd(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                               int num_seqs, const int32_t* cu_seqlens_host, int total_tokens,
                               int max_seqlen, int hq, int hkv, int head_dim, float softmax_scale,
                               hyd_dtype dt, void* o, float* lse, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
    return fwd_impl(q, k, v, cu_seqlens, num_seqs, cu_seqlens_host, nullptr, nullptr, false, total_tokens,
                    max_seqlen, hq, hkv, head_dim, softmax_scale, dt, o, lse, workspace, workspace_bytes,
                    hip_stream);
}

hyd_status hyd_varlen_attn_fwd_rope(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                                    int num_seqs, const int32_t* cu_seqlens_host, int total_tokens,
                                    int max_seqlen, int hq, int hkv, int head_dim, float softmax_scale,
                                    float rope_base, hyd_dtype dt, void* o, float* lse, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
    if (!(rope_base > 1.f)) return HYD_ERR_SHAPE;
    return fwd_impl(q, k, v, cu_seqlens, num_seqs, cu_seqlens_host, nullptr, nullptr, false, total_tokens,
                    max_seqlen, hq, hkv, head_dim, softmax_scale, dt, o, lse, workspace, workspace_bytes,
                    hip_stream, rope_base);
}

hyd_status hyd_varlen_attn_bwd_rope(const void* q, const void* k, const void* v, const void* o, const float* lse,
                                    const void* d_o, const int32_t* cu_seqlens, int num_seqs,
                                    const int32_t* cu_seqlens_host, int total_tokens, int max_seqlen, int hq,
                                    int hkv, int head_dim, float softmax_scale, float rope_base, hyd_dtype dt,
                                    void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                                    void* hip_stream) {
    if (!(rope_base > 1.f)) return HYD_ERR_SHAPE;
    return bwd_impl(q, k, v, o, lse, d_o, cu_seqlens, num_seqs, cu_seqlens_host, nullptr, nullptr, false,
                    total_tokens, max_seqlen, hq, hkv, head_dim, softmax_scale, dt, dq, dk, dv, workspace,
                    workspace_bytes, hip_stream, rope_base);
}

size_t hyd_varlen_attn_fwd_noalloc_max_workspace(void) { return kScratchBytes; }

hyd_status hyd_varlen_attn_fwd_noalloc(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                                       int num_seqs, const int32_t* cu_seqlens_host, int total_tokens,
                                       int max_seqlen, int hq, int hkv, int head_dim, float softmax_scale,
                                       hyd_dtype dt, void* o, float* lse, void* hip_stream) {
    // sizes first (no HIP call yet): the forward's workspace for these sizes must fit the array
    if (total_tokens < 0 || num_seqs < 0) return HYD_ERR_SHAPE;
    if (hq <= 0 || hkv <= 0 || hq % hkv != 0) return HYD_ERR_HEADS;
    if (dt != HYD_BF16 && dt != HYD_FP32) return HYD_ERR_DTYPE;
    if (!head_dim_ok(dt, head_dim)) return HYD_ERR_HEADDIM;
    if (hyd_varlen_attn_workspace_bytes(total_tokens, num_seqs, hq, hkv, head_dim, dt, 0) > kScratchBytes)
        return HYD_ERR_WORKSPACE;
    // the rest of the argument checks, still before any HIP call (a stand-in for the workspace pointer)
    const hyd_status vs = validate_common(cu_seqlens, num_seqs, cu_seqlens_host, total_tokens, max_seqlen, hq, hkv, head_dim,
                                          dt, reinterpret_cast<const void*>(kAlign), kScratchBytes, false);
    if (vs != HYD_OK) return vs;
    if (total_tokens == 0 || num_seqs == 0) return HYD_OK;
    if (!q || !k || !v || !o || !lse) return HYD_ERR_NULL;
    DeviceInfo* dev = nullptr;
    const hyd_status ds = device_info(&dev);          // first call on a device: looks the array's address up
    if (ds != HYD_OK) return ds;
    return fwd_impl(q, k, v, cu_seqlens, num_seqs, cu_seqlens_host, nullptr, nullptr, false, total_tokens, max_seqlen,
                    hq, hkv, head_dim, softmax_scale, dt, o, lse, dev->scratch, kScratchBytes, hip_stream);
}

hyd_status hyd_varlen_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                               const void* d_o, const int32_t* cu_seqlens, int num_seqs,
                               const int32_t* cu_seqlens_host, int total_tokens, int max_seqlen, int hq,
                               int hkv, int head_dim, float softmax_scale, hyd_dtype dt, void* dq, void* dk,
                               void* dv, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return bwd_impl(q, k, v, o, lse, d_o, cu_seqlens, num_seqs, cu_seqlens_host, nullptr, nullptr, false,
                    total_tokens, max_seqlen, hq, hkv, head_dim, softmax_scale, dt, dq, dk, dv, workspace,
                    workspace_bytes, hip_stream);
}

hyd_status hyd_varlen_attn_fwd_range(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                                     int num_seqs, const int32_t* cu_seqlens_host, const int32_t* ranges,
                                     const int32_t* ranges_host, int total_tokens, int max_seqlen, int hq,
                                     int hkv, int head_dim, float softmax_scale, hyd_dtype dt, void* o,
                                     float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return fwd_impl(q, k, v, cu_seqlens, num_seqs, cu_seqlens_host, ranges, ranges_host, true, total_tokens,
                    max_seqlen, hq, hkv, head_dim, softmax_scale, dt, o, lse, workspace, workspace_bytes,
                    hip_stream);
}

hyd_status hyd_varlen_attn_bwd_range(const void* q, const void* k, const void* v, const void* o,
                                     const float* lse, const void* d_o, const int32_t* cu_seqlens,
                                     int num_seqs, const int32_t* cu_seqlens_host, const int32_t* ranges,
                                     const int32_t* ranges_host, int total_tokens, int max_seqlen, int hq,
                                     int hkv, int head_dim, float softmax_scale, hyd_dtype dt, void* dq,
                                     void* dk, void* dv, void* workspace, size_t workspace_bytes,
                                     void* hip_stream) {
    return bwd_impl(q, k, v, o, lse, d_o, cu_seqlens, num_seqs, cu_seqlens_host, ranges, ranges_host, true,
                    total_tokens, max_seqlen, hq, hkv, head_dim, softmax_scale, dt, dq, dk, dv, workspace,
                    workspace_bytes, hip_stream);
}

hyd_status hyd_attn_merge(const void* o_a, const float* lse_a, const void* o_b, const float* lse_b,
                          int total_tokens, int hq, int head_dim, hyd_dtype dt, void* o_out, float* lse_out,
                          void* hip_stream) {
    if (dt != HYD_BF16) return HYD_ERR_DTYPE;
    if (total_tokens < 0) return HYD_ERR_SHAPE;
    if (hq <= 0) return HYD_ERR_HEADS;
    if (!head_dim_ok(dt, head_dim)) return HYD_ERR_HEADDIM;
    if (total_tokens == 0) return HYD_OK;
    if (!o_a || !lse_a || !o_b || !lse_b || !o_out || !lse_out) return HYD_ERR_NULL;
    DeviceInfo* dev = nullptr;
    const hyd_status ds = device_info(&dev);
    if (ds != HYD_OK) return ds;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const long long rows = (long long)total_tokens * hq;
    {
        KernelTimer kt("merge_bf16", st);
        const dim3 mgrid((unsigned)((rows + 15) / 16));
        if (head_dim == 64)
            hipLaunchKernelGGL(hyd_merge_bf16_kernel<64>, mgrid, dim3(256), 0, st, static_cast<const uint16_t*>(o_a), lse_a,
                               static_cast<const uint16_t*>(o_b), lse_b, static_cast<uint16_t*>(o_out), lse_out, total_tokens, hq);
        else
            hipLaunchKernelGGL(hyd_merge_bf16_kernel<kHeadDim>, mgrid, dim3(256), 0, st, static_cast<const uint16_t*>(o_a), lse_a,
                               static_cast<const uint16_t*>(o_b), lse_b, static_cast<uint16_t*>(o_out), lse_out, total_tokens, hq);
    }
    return hipGetLastError() == hipSuccess ? HYD_OK : HYD_ERR_LAUNCH;
}

hyd_status hyd_rope_packed(const void* x, const int32_t* cu_seqlens, int num_seqs, int total_tokens, int heads,
                           int head_dim, float base, int inverse, hyd_dtype dt, void* out, void* hip_stream) {
    if (dt != HYD_BF16) return HYD_ERR_DTYPE;
    if (total_tokens < 0 || num_seqs < 0 || (num_seqs == 0 && total_tokens != 0) || !(base > 1.f)) return HYD_ERR_SHAPE;
    if (heads <= 0) return HYD_ERR_HEADS;
    if (!head_dim_ok(dt, head_dim)) return HYD_ERR_HEADDIM;
    if (total_tokens == 0) return HYD_OK;
    if (!x || !cu_seqlens || !out) return HYD_ERR_NULL;
    DeviceInfo* dev = nullptr;
    const hyd_status ds = device_info(&dev);
    if (ds != HYD_OK) return ds;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    {
        KernelTimer kt("rope_bf16", st);
        const dim3 rgrid((unsigned)((total_tokens + kRopeTok - 1) / kRopeTok));
        if (head_dim == 64)
            hipLaunchKernelGGL(hyd_rope_bf16_kernel<64>, rgrid, dim3(kRopeThreads), 0, st, static_cast<const uint16_t*>(x), cu_seqlens,
                               num_seqs, total_tokens, heads, log2((double)base), inverse != 0, static_cast<uint16_t*>(out));
        else
            hipLaunchKernelGGL(hyd_rope_bf16_kernel<kHeadDim>, rgrid, dim3(kRopeThreads), 0, st, static_cast<const uint16_t*>(x), cu_seqlens,
                               num_seqs, total_tokens, heads, log2((double)base), inverse != 0, static_cast<uint16_t*>(out));
    }
    return hipGetLastError() == hipSuccess ? HYD_OK : HYD_ERR_LAUNCH;
}

hyd_status hyd_varlen_attn_schedule_layout(int total_tokens, int num_seqs, int hq, int hkv, int head_dim, hyd_dtype dt,
                                           int is_bwd, int which, size_t* header_offset, size_t* items_offset,
                                           int* max_items, int* tile) {
    if (!header_offset || !items_offset || !max_items || !tile) return HYD_ERR_NULL;
    if (total_tokens < 0 || num_seqs < 0 || which < 0 || which > 1 || (which == 1 && !is_bwd)) return HYD_ERR_SHAPE;
    if (hq <= 0 || hkv <= 0 || hq % hkv != 0) return HYD_ERR_HEADS;
    if (dt != HYD_BF16 && dt != HYD_FP32) return HYD_ERR_DTYPE;
    if (!head_dim_ok(dt, head_dim)) return HYD_ERR_HEADDIM;
    const WsLayout w = is_bwd ? ws_layout(total_tokens, num_seqs, tile_kv(dt), tile_dq(dt), hq, hkv, head_dim, dt, true)
                              : ws_layout(total_tokens, num_seqs, tile_fwd(dt), tile_fwd(dt), hq, hkv, head_dim, dt, false);
    const SchedLayout& v = w.sched[which];
    *header_offset = v.hdr; *items_offset = v.items; *max_items = v.max_items;
    *tile = !is_bwd ? tile_fwd(dt) : (which == 0 ? tile_kv(dt) : tile_dq(dt));
    return HYD_OK;
}

hyd_status hyd_varlen_attn_schedule_status(const void* workspace, size_t workspace_bytes, int total_tokens, int num_seqs,
                                           int hq, int hkv, int head_dim, hyd_dtype dt, int is_bwd, void* hip_stream) {
    size_t hdr = 0, items = 0;
    int max_items = 0, tile = 0;
    const hyd_status ls = hyd_varlen_attn_schedule_layout(total_tokens, num_seqs, hq, hkv, head_dim, dt, is_bwd, 0, &hdr, &items,
                                                          &max_items, &tile);
    if (ls != HYD_OK) return ls;
    if (total_tokens == 0 || num_seqs == 0) return HYD_OK;
    if (!workspace || workspace_bytes < hyd_varlen_attn_workspace_bytes(total_tokens, num_seqs, hq, hkv, head_dim, dt, is_bwd))
        return HYD_ERR_WORKSPACE;
    int head[2] = {0, 0};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(head, static_cast<const char*>(workspace) + hdr, sizeof(head), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return HYD_ERR_LAUNCH;
    if (head[kHdrFlags] & kSchedBadSeqlens) return HYD_ERR_SEQLENS;
    if (head[kHdrFlags] & kSchedTooLong) return HYD_ERR_SHAPE;
    return HYD_OK;
}

void hyd_enable_kernel_timing(int on) {
    t_timing = on != 0;
    timed_clear();
}

int hyd_kernel_times(const char** names, float* ms, int cap) {
    int n = 0;
    for (auto& t : t_timed) {
        if (n >= cap) break;
        float dt = 0.f;
        if (hipEventSynchronize(t.e1) != hipSuccess || hipEventElapsedTime(&dt, t.e0, t.e1) != hipSuccess) dt = -1.f;
        names[n] = t.name;
        ms[n] = dt;
        ++n;
    }
    timed_clear();
    return n;
}

void hyd_set_wg_trace(void* device_records, int capacity_records) {
    t_trace.rec = static_cast<unsigned long long*>(device_records);
    t_trace.capacity = device_records ? capacity_records : 0;
}

}  // extern "C"
