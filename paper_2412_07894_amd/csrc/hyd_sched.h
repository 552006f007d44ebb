// Work-item schedule of the persistent attention kernels.
//
// A work item is (sequence s, level c) with 1 <= c <= n_s = ceil(L_s / tile).  The forward and
// the dQ kernel read it as query tile c-1, whose causal span is c key tiles; the dK/dV kernel
// reads it as key tile n_s - c, which c query tiles attend to.  Either way the item's cost is
// proportional to c: the quadratic attention cost of a sequence (paper Sec. 2.1: cost is the sum
// of S_i^2; App. C.2: the quadratic term of T(l,P)) split into a ramp 1..n_s.  The prelude kernel
// writes the items in order of decreasing c.  Persistent workgroups then take items from the
// front of that list through atomic cursors, so the next-longest item always goes to the first
// workgroup that becomes free: longest-processing-time-first list scheduling.
//
// Heads multiply the items.  To keep the workgroups of one XCD (which share an L2) on the same
// K/V heads, the (item, head) space is split into 8 queues, one per XCD; a workgroup drains the
// queue of the XCD it runs on and then steals from the others, so every launch ends with all
// queues empty and no workgroup waits on another.
#pragma once
#include "hyd_device.h"
#include "hyd_rope_regs.h"

namespace hyd {

constexpr int kQueues = 8;

constexpr int kHdrInts = 64;
// header (ints): [0] n_items, [1] kSched* flags about cu_seqlens as the prelude saw it,
// [8 + 8*k + x] cursor of queue x of kernel k (k = 0 fwd, 1 dK/dV, 2 dQ); the rest is zeroed by
// the prelude and free for the kernels of the call ([40] of the dK/dV schedule: max |dO|)
constexpr int kHdrCursor = 8;
constexpr int kHdrFlags = 1;
constexpr int kSchedTooLong = 1;          // a sequence is longer than max_seqlen: its tiles beyond that bound got no item
constexpr int kSchedBadSeqlens = 2;       // cu_seqlens does not start at 0, does not end at T, or decreases

struct SchedView {            // device pointers into the workspace (all int32)
    int* hdr;                 // kHdrInts
    int* lev;                 // 3 * (n_lev + 2): level arrays, used instead of LDS when n_lev is large
    int* order;               // n_seq: sequence index by rank (more tiles first, then arrival)
    int* items;               // 4 * max_items : records (s, c, first packed row, length), decreasing c
    int n_lev;                // upper bound on tiles per sequence
    int max_items;
};

struct HeadMap {              // how (item, head) pairs are spread over the queues
    int striped;              // 0: heads partitioned over the queues; 1: items striped
    int heads;                // heads per item (Hq for fwd/dQ, Hkv for dK/dV)
    int hpq;                  // partitioned: heads per queue
    int group;                // partitioned: consecutive work indices share group-size heads
};

// In-place inclusive scan of v[0..n) by ONE wave (all 64 lanes call it; n arbitrary): every lane
// sums a contiguous chunk, the chunk sums are scanned across the lanes, each lane rewrites its chunk.
__device__ __forceinline__ void wave_inclusive_scan(int* v, int n, int lane) {
    const int chunk = (n + 63) / 64;
    const int lo = lane * chunk, hi = min(n, lo + chunk);
    __threadfence_block();                 // v was written by other lanes of this wave
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += v[i];
    int run = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(run, d, 64);
        if (lane >= d) run += up;
    }
    run -= sum;
    for (int i = lo; i < hi; ++i) { run += v[i]; v[i] = run; }
    __threadfence_block();                 // and is read by other lanes next
}

constexpr int kPreludeThreads = 1024;
constexpr int kPreludeLdsLev = 4096;      // levels whose arrays fit the kernel's LDS

// Builds the item list for tile size `tile` and clears the cursors; one workgroup per list
// (blockIdx.x = 0: tile0 -> sv0, blockIdx.x = 1: tile1 -> sv1), so the two lists of the backward
// come from one launch.  n_lev* bounds the tiles per sequence (from the caller's max_seqlen).
// Order among items of equal cost: by sequence rank (arrival order among equals), which is
// unspecified (it never changes a result: every output element has exactly one producer).
// With rope_tab != NULL the first workgroup also fills the rotary frequency table of the call
// (half_d entries, see hyd_rope_regs.h).
__global__ void __launch_bounds__(kPreludeThreads) hyd_schedule_prelude(const int32_t* __restrict__ cu, int nseq, int T,
                                                                       int tile0, SchedView sv0, int tile1, SchedView sv1,
                                                                       double* rope_tab, int half_d, double log2_base) {
    if (rope_tab && blockIdx.x == 0) rope_table_fill(rope_tab, half_d, log2_base, threadIdx.x, kPreludeThreads);
    __shared__ int lds_lev[3 * (kPreludeLdsLev + 2)];
    const bool second = blockIdx.x != 0;
    const int tile = second ? tile1 : tile0;
    const SchedView sv = second ? sv1 : sv0;
    const int tid = threadIdx.x;
    const int nl = sv.n_lev;
    int* lev = nl <= kPreludeLdsLev ? lds_lev : sv.lev;
    int* hist = lev;                       // [n]: sequences with exactly n tiles; later the arrival counters
    int* cnt = lev + (nl + 2);             // [r]: sequences with >= nl - r tiles (levels in reversed order)
    int* offs = lev + 2 * (nl + 2);        // [r]: list position after level nl - r
    for (int i = tid; i < nl + 2; i += kPreludeThreads) hist[i] = 0;
    for (int i = tid; i < kHdrInts; i += kPreludeThreads) sv.hdr[i] = 0;
    __syncthreads();
    int flags = (tid == 0 && (cu[0] != 0 || cu[nseq] != T)) ? kSchedBadSeqlens : 0;
    for (int s = tid; s < nseq; s += kPreludeThreads) {
        const int L = cu[s + 1] - cu[s];
        if (L < 0) flags |= kSchedBadSeqlens;
        if (L > 0 && (L + tile - 1) / tile > nl) flags |= kSchedTooLong;
        const int n = min((L + tile - 1) / tile, nl);
        if (n > 0) atomicAdd(&hist[n], 1);
    }
    if (flags) atomicOr(&sv.hdr[kHdrFlags], flags);
    __syncthreads();
    if (tid < 64) {
        // cnt[r] = sum_{n >= nl - r} hist[n]; offs = inclusive scan of cnt
        for (int r = tid; r < nl; r += 64) cnt[r] = hist[nl - r];
        wave_inclusive_scan(cnt, nl, tid);
        for (int r = tid; r < nl; r += 64) offs[r] = cnt[r];
        wave_inclusive_scan(offs, nl, tid);
    }
    __syncthreads();
    const int n_items = nl > 0 ? min(offs[nl - 1], sv.max_items) : 0;
    if (tid == 0) sv.hdr[0] = n_items;
    for (int i = tid; i < nl + 2; i += kPreludeThreads) hist[i] = 0;
    __syncthreads();
    // rank of a sequence with n tiles = (#sequences with more tiles) + arrival order among equals
    for (int s = tid; s < nseq; s += kPreludeThreads) {
        const int L = cu[s + 1] - cu[s];
        const int n = min((L + tile - 1) / tile, nl);
        if (n == 0) continue;
        const int more = (n < nl) ? cnt[nl - (n + 1)] : 0;
        sv.order[more + atomicAdd(&hist[n], 1)] = s;
    }
    __syncthreads();
    // Level c (reversed index r = nl - c) holds the sequences of rank < cnt[r] at the list
    // positions [offs[r] - cnt[r], offs[r]): one thread per position finds its level by bisection.
    for (int pos = tid; pos < n_items; pos += kPreludeThreads) {
        int lo = 0, hi = nl - 1;               // first r with offs[r] > pos
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (offs[mid] > pos) hi = mid; else lo = mid + 1;
        }
        const int s = sv.order[pos - (offs[lo] - cnt[lo])];
        const int a = cu[s];
        int* rec = sv.items + 4 * pos;
        rec[0] = s; rec[1] = nl - lo; rec[2] = a; rec[3] = cu[s + 1] - a;
    }
}

// Number of work indices of queue x.
__device__ __forceinline__ int queue_size(const HeadMap& hm, int n_items, int x) {
    if (hm.striped) return ((n_items - x + kQueues - 1) / kQueues) * hm.heads;
    return n_items * hm.hpq;
}

// Work index w of queue x -> (item index, head).  A partitioned queue walks the item list in
// chunks of chunk_items() items (the list is ordered by decreasing cost, so a chunk holds items of
// similar cost, in a long sequence neighbouring tiles) and, inside a chunk, one head group after
// the other.  The 32 workgroups of an XCD then sit on neighbouring tiles of ONE KV head (times its
// group's query heads) and share the K/V (or Q/dO) tiles they stream in their L2; with the heads
// interleaved per item, a queue with several groups (MHA: every head is its own group) split
// its workgroups over all of them and shared each stream among a fifth as many.  Walking whole
// groups one after the other would share as well but starts the last group's longest items late,
// which unbalances the end of a short launch; chunks keep the order longest-first up to a window
// of one chunk, an eighth of the list at most.  Measured (one process, both orders alternating):
// the MHA configuration 3 gains 4-6 % in every kernel with chunks of 64, the single-buffer
// configuration 2 (67 items in the forward's list) loses 10 % with whole groups or chunks of 64
// and nothing with chunks of 8-16; the GQA configurations, one group per queue, do not change.
__device__ __forceinline__ int chunk_items(int n_items) { return min(64, max(8, n_items >> 3)); }
__device__ __forceinline__ void decode_work(const HeadMap& hm, int n_items, int x, int w, int& item, int& head) {
    if (hm.striped) {
        item = x + kQueues * (w / hm.heads);
        head = w % hm.heads;
    } else {
        const int chunk = chunk_items(n_items);
        const int per_chunk = chunk * hm.hpq;              // work indices of a full chunk
        const int ck = w / per_chunk, r = w - ck * per_chunk;
        const int first = ck * chunk;
        const int per_group = min(chunk, n_items - first) * hm.group;
        const int grp = r / per_group, r2 = r - grp * per_group;
        item = first + r2 / hm.group;
        head = (x + kQueues * grp) * hm.group + r2 % hm.group;
    }
}

// Persistent-workgroup work fetch.  Thread 0 takes work indices from the queue of its XCD through
// an atomic cursor, moving on to the next queue when one is exhausted, resolves an index to
// (item, head), fetches the item's 16-byte record and leaves the result in LDS for the workgroup.
//
// The chain "cursor atomic -> item record" is two dependent trips to memory, as long as a whole
// short item, so the atomic is taken off the critical path: the one for item k+1 is issued when
// item k begins (in next(), right after the barrier that ends item k-1) and its result is only
// looked at when item k ends, an item's duration later.  What remains at the end of an item is
// one trip for the record.  A workgroup thus holds one claimed item ahead of the one it works on
// (holding two, with the record fetched early as well, costs more balance at the end of a launch
// than it saves).  Only when a queue runs dry (eight times in a workgroup's life) is a claim
// repeated on the next queue synchronously.  Every workgroup ends when all queues are empty
// (the cursors only grow).
struct WorkItem { int seq, lev, head, row0, len; };
constexpr int kSlotInts = 16;          // two buffers of 8 ints
typedef __attribute__((ext_vector_type(4))) int i32x4;

struct WorkFetcher {
    int cur;          // slot buffer holding the current item (all threads)
    // the rest is thread 0's
    int queue;        // queue the next claim goes to
    int tried;        // queues found empty so far
    int n_items;
    int claim_q;      // queue of the claim in flight
    int claim_w;      // its result (the atomic's return value; no use of it until one item later)
    int nxt_item;     // next item: index (-1: none), head, and its record in flight
    int nxt_head;
    i32x4 nxt_rec;

    __device__ __forceinline__ void issue_claim(const HeadMap& hm, int* cursors) {
        claim_q = queue;
        const bool open = tried < kQueues && queue_size(hm, n_items, queue) > 0;
        claim_w = open ? atomicAdd(&cursors[queue], 1) : 0x7fffffff;
    }
    // Turns the claim in flight into (item, head) of the next item and requests its record.
    __device__ __forceinline__ void resolve(const HeadMap& hm, int* cursors, const int* __restrict__ items) {
        int q = claim_q, w = claim_w;
        nxt_item = -1;
        nxt_head = 0;
        while (tried < kQueues) {
            if (w < queue_size(hm, n_items, q)) {
                decode_work(hm, n_items, q, w, nxt_item, nxt_head);
                break;
            }
            if (q == queue) {                       // that queue is exhausted: on to the next one
                queue = (queue + 1) & (kQueues - 1);
                ++tried;
                if (tried >= kQueues) break;
            }
            q = queue;
            w = queue_size(hm, n_items, q) > 0 ? atomicAdd(&cursors[q], 1) : 0x7fffffff;
        }
        if (nxt_item >= 0) nxt_rec = *reinterpret_cast<const i32x4*>(items + 4 * nxt_item);
    }
    __device__ __forceinline__ void publish(int* buf) const {
        buf[0] = nxt_item;
        buf[1] = nxt_head;
        if (nxt_item >= 0) { buf[2] = nxt_rec[0]; buf[3] = nxt_rec[1]; buf[4] = nxt_rec[2]; buf[5] = nxt_rec[3]; }
    }
    __device__ __forceinline__ bool read(const int* buf, WorkItem& w) const {
        if (buf[0] < 0) return false;
        w.head = buf[1]; w.seq = buf[2]; w.lev = buf[3]; w.row0 = buf[4]; w.len = buf[5];
        return true;
    }
    // `slot`: kSlotInts ints of LDS.  All threads must call first/next (each contains a barrier).
    __device__ __forceinline__ bool first(const HeadMap& hm, const int* __restrict__ hdr, int* cursors,
                                          const int* __restrict__ items, int* slot, WorkItem& w) {
        cur = 0;
        if (threadIdx.x == 0) {
            queue = (__smid() >> 6) & (kQueues - 1);     // XCC id of this workgroup
            tried = 0;
            n_items = hdr[0];
            issue_claim(hm, cursors);
            resolve(hm, cursors, items);
            publish(slot);
        }
        __syncthreads();
        if (threadIdx.x == 0) issue_claim(hm, cursors);  // for the item after the first
        return read(slot, w);
    }
    __device__ __forceinline__ bool next(const HeadMap& hm, int* cursors, const int* __restrict__ items,
                                         int* slot, WorkItem& w) {
        if (threadIdx.x == 0) {
            resolve(hm, cursors, items);                 // the claim issued when this item began
            publish(slot + 8 * (cur ^ 1));
        }
        __syncthreads();        // the next item is visible; everybody is done with the LDS tiles
        if (threadIdx.x == 0) issue_claim(hm, cursors);  // for the item after the next
        cur ^= 1;
        return read(slot + 8 * cur, w);
    }
};

// Optional per-workgroup trace record: {kernel id << 32 | CU key, start, end, items}.
struct WgTrace {
    unsigned long long* rec;      // nullptr: off
    int capacity;
};
__device__ __forceinline__ void trace_write(const WgTrace& tr, int kernel_id, unsigned long long t0,
                                            unsigned long long n_items_done) {
    if (tr.rec && threadIdx.x == 0) {
        const int per_kernel = tr.capacity / 3;
        const int idx = kernel_id * per_kernel + blockIdx.x;
        if ((int)blockIdx.x < per_kernel) {
            unsigned long long* r = tr.rec + 4 * (size_t)idx;
            r[0] = ((unsigned long long)kernel_id << 32) | (unsigned long long)__smid();
            r[1] = t0;
            r[2] = wall_clock64();
            r[3] = n_items_done;
        }
    }
}

}  // namespace hyd
