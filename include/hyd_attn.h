/*
 * hyd_attn.h - C ABI of the MI355X (gfx950) packed variable-length causal self-attention library.
 *
 * The operation is the per-replica hot path of Hydraulis (arXiv 2412.07894): several sequences
 * are concatenated ("packed") into one buffer of T tokens and attention is applied to each
 * sequence on its own, so the mask is block diagonal (and causal inside each block) and the cost
 * is the sum of S_i^2 over the packed sequences instead of (sum S_i)^2 (paper Sec. 2.1, packing
 * paragraph; Sec. 6.1 "Solving for one V": the latency of a packed buffer is the sum over its
 * sequences).  One forward plus one backward over a packed buffer is the unit of work that the
 * paper's latency model T(l,P) prices (Sec. 6.1; App. C.2: the quadratic term is attention).
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never allocates,
 *     frees or keeps them, never synchronises the device and enqueues work only on `hip_stream`
 *     (a hipStream_t passed as void*; NULL is the default stream).  Results are valid once the
 *     stream has executed the work enqueued by the call; `workspace` must stay alive until then.
 *   - Layouts are contiguous, token major: Q, O, dO, dQ are [T][Hq][d]; K, V, dK, dV are
 *     [T][Hkv][d]; LSE is float [Hq][T] (natural log).  dtype HYD_BF16: 2-byte bfloat16 elements;
 *     dtype HYD_FP32: 4-byte float elements; head_dim 64 or 128 for both (the bf16 kernels are
 *     laid out for 128; at 64 they run the same tiles with half the contraction steps and half
 *     the output blocks).  Outputs have the dtype of the inputs and are fully overwritten.
 *   - Tiles are fetched through 32-bit buffer resources based at the start of a sequence, so
 *     max_seqlen * Hq * head_dim * element size must be below 4 GiB (2 GiB for bf16 with
 *     head_dim 64; HYD_ERR_SHAPE otherwise).
 *   - cu_seqlens is int32[num_seqs+1] ON THE DEVICE: cu[0] = 0, cu[num_seqs] = T, non-decreasing;
 *     sequence s owns packed rows [cu[s], cu[s+1]).  Empty sequences are legal.  Every token
 *     belongs to exactly one sequence.  `cu_seqlens_host` is an optional HOST copy of the same
 *     array (may be NULL); when given it is validated before anything is enqueued.
 *   - Query head h reads KV head h / (Hq/Hkv) (grouped-query attention with contiguous groups).
 *   - Masking is always causal in LOCAL positions: key j of a sequence is visible to query i of
 *     the same sequence iff j <= i.  No dropout, bias, window or positional encoding.
 *   - Errors are return codes.  All argument validation happens before the first HIP call, so
 *     every HYD_ERR_* below except HYD_ERR_ARCH and HYD_ERR_LAUNCH can be provoked on a host
 *     without a GPU.  On error nothing has been enqueued.
 *   - Calls are re-entrant as long as concurrent calls use distinct workspaces.
 */
#ifndef HYD_ATTN_H
#define HYD_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HYD_OK = 0,
    HYD_ERR_NULL = 1,       /* a required pointer is NULL */
    HYD_ERR_SHAPE = 2,      /* negative sizes, max_seqlen out of range or below the longest sequence */
    HYD_ERR_DTYPE = 3,      /* dtype is neither HYD_BF16 nor HYD_FP32 */
    HYD_ERR_HEADS = 4,      /* hq <= 0, hkv <= 0 or hq % hkv != 0 */
    HYD_ERR_HEADDIM = 5,    /* head_dim not supported for this dtype */
    HYD_ERR_SEQLENS = 6,    /* host cu_seqlens does not start at 0, end at T or is decreasing */
    HYD_ERR_WORKSPACE = 7,  /* workspace NULL, misaligned (256 B) or smaller than required */
    HYD_ERR_ARCH = 8,       /* the current device is not gfx950 */
    HYD_ERR_LAUNCH = 9,     /* a HIP launch or query failed */
    HYD_ERR_INFEASIBLE = 10,/* planning calls (hyd_plan.h): the constraints admit no solution */
    HYD_ERR_RANGE = 11      /* range variants: a range is misaligned or has end < begin */
} hyd_status;

typedef enum { HYD_BF16 = 0, HYD_FP32 = 1 } hyd_dtype;

/* Human-readable name of a status code (static storage; never NULL). */
const char* hyd_status_string(hyd_status st);

/*
 * Bytes of device workspace that hyd_varlen_attn_fwd (is_bwd = 0) or hyd_varlen_attn_bwd
 * (is_bwd = 1) needs for these sizes.  The workspace holds the work-item schedule (the list of
 * (sequence, tile) items ordered by decreasing cost, and the queue cursors of the persistent
 * workgroups) and, for the backward, float vectors [Hq][T] of row statistics (D = rowsum(dO * O)
 * and LSE in base-2 units, negated, in the forms the two kernels consume) plus, for bf16, fp16
 * copies of Q, dO and K (2 * T * (2 Hq + Hkv) * head_dim bytes); the contents are private to the
 * library.  Returns 0 for invalid arguments.  Pure host arithmetic: no HIP call.
 */
size_t hyd_varlen_attn_workspace_bytes(int total_tokens, int num_seqs, int hq, int hkv,
                                       int head_dim, hyd_dtype dt, int is_bwd);

/*
 * Forward (paper Sec. 2.1: block-diagonal "varlen" attention; causal because the models are
 * decoder-only, Sec. 8.1).  For every sequence s, query head h, local row i:
 *     s_ij = softmax_scale * <Q_i, K_j>, j <= i;   P_i. = softmax_j(s_i.);
 *     O_i = sum_j P_ij V_j;                        LSE_i = ln sum_j exp(s_ij).
 *
 *   q, k, v          device, inputs (layouts above)
 *   cu_seqlens       device int32[num_seqs+1]
 *   cu_seqlens_host  host copy or NULL
 *   total_tokens     T >= 0;  max_seqlen: an upper bound on the longest sequence (1..T)
 *   o, lse           device, outputs; rows of o / entries of lse are written for every token
 *   workspace        device, >= hyd_varlen_attn_workspace_bytes(..., 0) bytes, 256-byte aligned;
 *                    contents need not be initialised and are clobbered
 * T == 0 or num_seqs == 0 is a no-op returning HYD_OK.
 */
hyd_status hyd_varlen_attn_fwd(const void* q, const void* k, const void* v,
                               const int32_t* cu_seqlens, int num_seqs,
                               const int32_t* cu_seqlens_host,
                               int total_tokens, int max_seqlen, int hq, int hkv, int head_dim,
                               float softmax_scale, hyd_dtype dt,
                               void* o, float* lse,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of the above for an upstream gradient dO of O (LSE carries no gradient).  One forward
 * and one backward are the paper's unit "a single forward and backward propagation" (Sec. 6.1).
 *     dP_ij = <dO_i, V_j>;  D_i = <dO_i, O_i>;  dS_ij = P_ij (dP_ij - D_i),  P_ij = exp(s_ij - LSE_i)
 *     dQ_i = scale * sum_{j<=i} dS_ij K_j
 *     dK_j = scale * sum_{h in group} sum_{i>=j} dS_ij Q_i
 *     dV_j =         sum_{h in group} sum_{i>=j} P_ij dO_i
 *
 *   q, k, v, o, lse  device, the forward's inputs and outputs (o and lse as the forward wrote them)
 *   d_o              device, [T][Hq][d], same dtype
 *   dq, dk, dv       device, outputs, fully overwritten (no atomics: bitwise reproducible)
 *   workspace        device, >= hyd_varlen_attn_workspace_bytes(..., 1) bytes, 256-byte aligned
 * Four kernels are enqueued after the schedule prelude (one launch for both item lists): row
 * statistics (D = rowsum(dO * O), the largest |dO| of each row and of the tensor); fp16 copies of
 * Q, K and dO; dK/dV (one work item per (sequence, key tile, KV head), looping over the group's
 * query heads); dQ (one work item per (sequence, query tile, query head)).
 *
 * Arithmetic of the bf16 path: the tile products run on the fp16 matrix instructions with fp32
 * accumulation, so that the factors formed in registers (P, dS) keep 11 significant bits.  bf16
 * inputs convert to fp16 exactly for magnitudes in [2^-14, 65504]; Q, K or V values beyond 65504
 * become infinite (the gradients are then non-finite), values below 2^-14 keep an absolute
 * accuracy of 2^-25.  dO may have any scale: it is brought into range by powers of two (one per
 * tensor for dK and dV, one per row for dQ) that are undone in the results.  D is formed from the
 * o that is passed in: where o has been rounded to bf16, dQ and dK carry that rounding
 * (<dO_i, delta O_i> enters every dS_ij of the row), whatever the arithmetic of the kernels.
 */
hyd_status hyd_varlen_attn_bwd(const void* q, const void* k, const void* v, const void* o,
                               const float* lse, const void* d_o,
                               const int32_t* cu_seqlens, int num_seqs,
                               const int32_t* cu_seqlens_host,
                               int total_tokens, int max_seqlen, int hq, int hkv, int head_dim,
                               float softmax_scale, hyd_dtype dt,
                               void* dq, void* dk, void* dv,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Forward and backward with the rotary position embedding of Q applied inside the kernels.
 * Packing requires positions that restart in every packed sequence (paper Sec. 2.1, the packing
 * paragraph); the kernels know the local position of every query row, so Q needs no pass of its
 * own through HBM: `q` is the UNROTATED Q, rotated as a work item picks its rows up (pairing,
 * angles and `rope_base` as in hyd_rope_packed below, position = row index inside its sequence).
 * `k` must already be rotated (one hyd_rope_packed call per layer: every query tile of a sequence
 * streams K again, rotating it there would repeat the work).  The backward returns dQ for the
 * unrotated Q (it turns the gradient back before writing it) and dK for the rotated K that was
 * passed in (apply hyd_rope_packed with inverse = 1 to it for the gradient of the unrotated K).
 * bf16 only (else HYD_ERR_DTYPE); rope_base must exceed 1 (else HYD_ERR_SHAPE); everything else
 * as hyd_varlen_attn_fwd / hyd_varlen_attn_bwd, including the workspace sizes.
 */
hyd_status hyd_varlen_attn_fwd_rope(const void* q, const void* k, const void* v,
                                    const int32_t* cu_seqlens, int num_seqs,
                                    const int32_t* cu_seqlens_host,
                                    int total_tokens, int max_seqlen, int hq, int hkv, int head_dim,
                                    float softmax_scale, float rope_base, hyd_dtype dt,
                                    void* o, float* lse,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);
hyd_status hyd_varlen_attn_bwd_rope(const void* q, const void* k, const void* v, const void* o,
                                    const float* lse, const void* d_o,
                                    const int32_t* cu_seqlens, int num_seqs,
                                    const int32_t* cu_seqlens_host,
                                    int total_tokens, int max_seqlen, int hq, int hkv, int head_dim,
                                    float softmax_scale, float rope_base, hyd_dtype dt,
                                    void* dq, void* dk, void* dv,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * What the schedule prelude of the last forward (is_bwd = 0) or backward (is_bwd = 1) call on
 * `workspace` saw in the DEVICE cu_seqlens.  The entry points above cannot look at device memory
 * without stalling the stream, so with cu_seqlens_host == NULL they trust the caller: a sequence
 * longer than max_seqlen gets work items only for its first ceil(max_seqlen / tile) tiles (the
 * rest of its outputs is left unwritten), and a cu_seqlens that does not start at 0, end at
 * total_tokens or that decreases gives undefined results inside the buffers.  This call copies
 * the prelude's findings back - it SYNCHRONISES `hip_stream` - and returns HYD_ERR_SHAPE for
 * the first condition, HYD_ERR_SEQLENS for the second, HYD_OK otherwise.  Same size arguments
 * as the call it checks.  Errors of its own: HYD_ERR_WORKSPACE, the argument errors, HYD_ERR_LAUNCH.
 */
hyd_status hyd_varlen_attn_schedule_status(const void* workspace, size_t workspace_bytes,
                                           int total_tokens, int num_seqs, int hq, int hkv,
                                           int head_dim, hyd_dtype dt, int is_bwd, void* hip_stream);

/*
 * Where a schedule sits inside a workspace, for tools that inspect it (pure host arithmetic).
 * which = 0: the forward's list (is_bwd = 0) or the dK/dV kernel's (is_bwd = 1); which = 1: the
 * dQ kernel's (is_bwd = 1 only).  At header_offset: int32[64], [0] = number of items n.  At
 * items_offset: n records of four int32 (sequence, level c, first packed row of the sequence,
 * length of the sequence), by decreasing level (paper Sec. 2.1: the cost of a sequence is
 * quadratic; level c of a sequence is its tile with c tiles of causal work, 1 <= c <=
 * ceil(length / *tile)); at most *max_items records.
 */
hyd_status hyd_varlen_attn_schedule_layout(int total_tokens, int num_seqs, int hq, int hkv,
                                           int head_dim, hyd_dtype dt, int is_bwd, int which,
                                           size_t* header_offset, size_t* items_offset,
                                           int* max_items, int* tile);

/*
 * Forward without a workspace argument, for callers that cannot allocate device memory or carry a
 * workspace around (code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation): same computation and results as hyd_varlen_attn_fwd, with the schedule kept in a
 * fixed array inside the library (hyd_varlen_attn_fwd_noalloc_max_workspace() bytes per GPU,
 * held until the process ends).  It calls no hipMalloc / hipFree and no allocating routine.
 * Sizes whose forward workspace (hyd_varlen_attn_workspace_bytes(..., 0)) exceeds that array
 * are rejected with HYD_ERR_WORKSPACE before any HIP call; 2 MiB cover, for example, one million
 * tokens in 65536 sequences.  All calls on one GPU share the one array: two calls whose kernels
 * overlap in time (different streams, or different host threads) race on it, so serialise them.
 * Argument checks, errors and stream semantics otherwise as hyd_varlen_attn_fwd.
 */
hyd_status hyd_varlen_attn_fwd_noalloc(const void* q, const void* k, const void* v,
                                       const int32_t* cu_seqlens, int num_seqs,
                                       const int32_t* cu_seqlens_host,
                                       int total_tokens, int max_seqlen, int hq, int hkv, int head_dim,
                                       float softmax_scale, hyd_dtype dt,
                                       void* o, float* lse, void* hip_stream);
size_t hyd_varlen_attn_fwd_noalloc_max_workspace(void);

/*
 * Range variants: the building block of context parallelism (CP, one axis of the paper's
 * <TP, PP, CP> schemes, Sec. 2.1 and App. C.1).  Under CP a device holds one chunk of every
 * sequence's queries while the key/value chunks visit it one after the other; each visit
 * computes the attention of a query range against a key range, and the partial results are
 * merged by the log-sum-exp rule (hyd_attn_merge).  The calls below do one such visit for all
 * sequences of a packed buffer; the buffers keep the layout of the plain calls (whole
 * sequences, T rows), the ranges select what is computed.
 *
 *   ranges           device int32[4 * num_seqs]: per sequence (q_begin, q_end, kv_begin, kv_end)
 *                    in LOCAL positions of the sequence.  Begins are multiples of
 *                    HYD_RANGE_ALIGN; an end is a multiple of it too, or lies at or past the end
 *                    of the sequence (it is then capped there).  end >= begin >= 0.  An empty
 *                    range is allowed.
 *   ranges_host      host copy or NULL; when given, the rules above are checked (HYD_ERR_RANGE;
 *                    exactly if cu_seqlens_host is given too, else against max_seqlen).  Ranges
 *                    that break the rules without a host copy give wrong values for the
 *                    sequences concerned, never an access outside the buffers.
 *   dt               HYD_BF16 only (HYD_ERR_DTYPE otherwise)
 * Forward: for local row i of the query range, over the keys j of the key range with j <= i,
 *     LSE_i = ln sum_j exp(s_ij),  O_i = sum_j exp(s_ij - LSE_i) V_j;
 * a row that sees no such key gets O_i = 0 and LSE_i = -inf.  Rows outside the query range are
 * NOT written.
 */
#define HYD_RANGE_ALIGN 256

hyd_status hyd_varlen_attn_fwd_range(const void* q, const void* k, const void* v,
                                     const int32_t* cu_seqlens, int num_seqs,
                                     const int32_t* cu_seqlens_host,
                                     const int32_t* ranges, const int32_t* ranges_host,
                                     int total_tokens, int max_seqlen, int hq, int hkv, int head_dim,
                                     float softmax_scale, hyd_dtype dt,
                                     void* o, float* lse,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of one visit.  o and lse are the MERGED forward results of the rows (their full
 * softmax over all visible keys), so that P_ij = exp(s_ij - LSE_i) and D_i = <dO_i, O_i> are the
 * true ones; with them
 *     dq rows of the query range = scale * sum_{j in key range, j <= i} dS_ij K_j
 *     dk / dv rows of the key range = the sums of hyd_varlen_attn_bwd restricted to the rows i of
 *                                  the query range.
 * Summed over a partition of the keys (dq) or of the queries (dk, dv) they give the gradients
 * of the plain call; the sum is the caller's (each call rounds its partial to the buffer's
 * dtype).  Rows of dq outside the query range and rows of dk / dv outside the key range are NOT
 * written.  Other arguments as hyd_varlen_attn_bwd / hyd_varlen_attn_fwd_range.
 */
hyd_status hyd_varlen_attn_bwd_range(const void* q, const void* k, const void* v, const void* o,
                                     const float* lse, const void* d_o,
                                     const int32_t* cu_seqlens, int num_seqs,
                                     const int32_t* cu_seqlens_host,
                                     const int32_t* ranges, const int32_t* ranges_host,
                                     int total_tokens, int max_seqlen, int hq, int hkv, int head_dim,
                                     float softmax_scale, hyd_dtype dt,
                                     void* dq, void* dk, void* dv,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Log-sum-exp merge of two partial results over the same T rows (all device pointers;
 * o_* [T][Hq][d] in dt, lse_* float [Hq][T], natural log):
 *     LSE = ln(exp(LSE_a) + exp(LSE_b)),  O = exp(LSE_a - LSE) O_a + exp(LSE_b - LSE) O_b.
 * A row whose LSE is -inf in one partial takes the other partial unchanged (whatever bits that
 * row of the -inf partial's O holds); -inf in both gives O = 0, LSE = -inf.  o_out / lse_out may
 * be the same buffers as either input pair (in-place accumulation over the visits).
 * HYD_BF16 only.  No workspace.
 */
hyd_status hyd_attn_merge(const void* o_a, const float* lse_a, const void* o_b, const float* lse_b,
                          int total_tokens, int hq, int head_dim, hyd_dtype dt,
                          void* o_out, float* lse_out, void* hip_stream);

/*
 * Rotary position embedding of a packed buffer, the position reset at every sequence start
 * (Sec. 2.1: packing requires that the positional embedding be adjusted so that a sequence keeps
 * the positions it would have alone; the paper's models, LLaMA 2, use rotary embeddings).  For
 * packed row t of sequence s, local position m = t - cu_seqlens[s], and pair i in [0, d/2) of
 * every head:
 *     angle = m * base^(-2 i / d)
 *     out[i]       = x[i] cos(angle) - x[i + d/2] sin(angle)
 *     out[i + d/2] = x[i + d/2] cos(angle) + x[i] sin(angle)
 * inverse != 0 negates the angle: the transpose of the rotation, which maps the gradient of the
 * rotated tensor to the gradient of the input.  Apply it to Q and K before the attention calls
 * and, inverted, to dQ and dK after the backward.
 *   x, out           device, [T][heads][d] in dt; out may be x (in place)
 *   cu_seqlens       device int32[num_seqs+1] as above
 *   base             > 1 (10000 for the paper's models)
 * HYD_BF16 only (head_dim 64 or 128).  No workspace; one kernel, bound by HBM.
 */
hyd_status hyd_rope_packed(const void* x, const int32_t* cu_seqlens, int num_seqs, int total_tokens,
                           int heads, int head_dim, float base, int inverse, hyd_dtype dt,
                           void* out, void* hip_stream);

/*
 * Timing hook for benchmarks.  While enabled (on != 0), every kernel that a later call of this
 * library enqueues from this host thread is bracketed with HIP events on the caller's stream and
 * appended to a per-thread list (at most 8192 launches; further ones are not recorded).  Nothing
 * is synchronised while recording.  hyd_kernel_times synchronises the recorded events, fills up to
 * `cap` entries of names[] (static strings) and ms[] (milliseconds) in launch order, empties the
 * list and returns the number of entries filled (0 when timing is off).  Enabling or disabling
 * also empties the list.  Off by default; when off the entry points enqueue nothing but their
 * kernels.
 */
void hyd_enable_kernel_timing(int on);
int  hyd_kernel_times(const char** names, float* ms, int cap);

/*
 * Per-workgroup busy-time instrumentation of the persistent kernels.  With a non-NULL device
 * buffer of `capacity_records` records registered here, every persistent workgroup of the later
 * fwd / bwd calls on this host thread writes one record of 4 x uint64:
 *     { kernel id (0 fwd, 1 dK/dV, 2 dQ) << 32 | physical CU key (XCC id, SE id, CU id),
 *       start clock, end clock, number of work items processed }
 * at index (kernel id * (capacity_records / 3) + workgroup); workgroups beyond capacity_records / 3
 * write nothing.  Pass NULL to switch it off.  The clock is the
 * constant-rate wall clock (100 MHz).  For measurement builds only: adds two clock reads and one
 * 32-byte store per workgroup.
 */
void hyd_set_wg_trace(void* device_records, int capacity_records);

#ifdef __cplusplus
}
#endif
#endif /* HYD_ATTN_H */
