/*
 * mtfm_hta.h -- C ABI of libmtfm_hta.so: grouped-query Hybrid Target Attention (HTA) over jagged
 * user-level aggregated samples, hand-written for AMD gfx950 (MI355X).
 *
 * The operation (Section 3.2.2, "Hybrid Target Attention Architecture"):
 *   full attention layer    A^(h)   = phi2(Q^(h)   K^(g)T (.) M  ) V^(g)      every token of a user is a query
 *   target attention layer  A_T^(h) = phi2(Q_T^(h) K^(g)T (.) M_T) V^(g)      queries = the user's target tokens,
 *                                                                            M_T = those rows of M, K/V = all tokens
 *   grouped-query heads: query head h (0-based) reads key/value head g = h / r, r = Hq / Hkv
 *                        (the paper's g = ceil(h/r) for 1-based h): consecutive query heads share a kv head.
 *   dynamic mask M (rules 1 and 3): history tokens are visible to every token, a target token only to
 *   itself.  The mask is never materialised: it is a function of (hist_len, token index).
 *   Heads are concatenated along the feature axis (A = A^1 || ... || A^H): the [token][head][d] layout.
 * Readings fixed where the paper is silent: phi2 is a row softmax over the visible keys (masked keys get
 * weight exactly 0); logits are multiplied by the explicit softmax_scale; lse is the natural-log
 * logsumexp of the scaled visible logits.
 *
 * Data layout.  A batch holds `batch` users packed back to back, no padding.  User b owns
 *   K/V rows  kv_offsets[b] .. kv_offsets[b+1]-1 :  hist_len[b] history tokens, then n_targets[b] target tokens
 *             (token order X = (H; T) of Section 3.2.1), so kv_offsets[b+1]-kv_offsets[b] = hist_len[b]+n_targets[b];
 *   Q rows    q_offsets[b] .. q_offsets[b+1]-1 :  the same tokens (full layer; q_offsets may alias kv_offsets)
 *             or only the n_targets[b] target tokens (target layer; q_offsets = prefix sums of n_targets).
 *   q, out, dout, dq : [total_q ][Hq ][head_dim]  row-major
 *   k, v, dk, dv     : [total_kv][Hkv][head_dim]  row-major
 *   lse              : [Hq][total_q] float32
 *
 * Pointers.  Every data pointer (q,k,v,out,lse,dout,dq,dk,dv, the four int32 arrays, workspace) is a
 * DEVICE pointer; `stream` is a hipStream_t passed as void* (NULL = the default stream).  The caller
 * owns all buffers.  The functions declared in this header never allocate or free device memory, never copy
 * to the host and never synchronise: a call validates its scalar arguments on the host, enqueues kernels on
 * `stream` and returns.  (The optional instrumentation of mtfm_hta_timing.h is separate and does block.)
 * Device-resident arrays are not validated (that would need a device-to-host copy); they must satisfy the
 * layout above, and hist_len[b] <= max_hist, n_targets[b] <= max_targets.
 *
 * Errors.  Every entry point returning int returns an mtfm_hta_status; on a non-zero status nothing
 * has been enqueued (except MTFM_HTA_ERR_LAUNCH, reported by the runtime after an enqueue), and
 * mtfm_hta_last_error() describes the problem.
 */
#ifndef MTFM_HTA_H
#define MTFM_HTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported with default visibility; everything else in the library is hidden */
#define MTFM_HTA_API __attribute__((visibility("default")))

typedef enum {
    MTFM_HTA_OK = 0,
    MTFM_HTA_ERR_INVALID_ARG = -1, /* null pointer, misaligned pointer, negative size, Hq % Hkv != 0, bad enum, scale <= 0 */
    MTFM_HTA_ERR_UNSUPPORTED = -2, /* head_dim / head-group shape this build has no kernel for */
    MTFM_HTA_ERR_WORKSPACE = -3,   /* workspace missing or smaller than mtfm_hta_workspace_bytes() */
    MTFM_HTA_ERR_LAUNCH = -4       /* the HIP runtime refused a launch */
} mtfm_hta_status;

/* element type of q, k, v, out, dout, dq, dk, dv */
enum { MTFM_HTA_BF16 = 0, /* bfloat16 storage, MFMA with fp32 accumulation; head_dim in {16, 32, 64, 128}.  A 16-wide
                             head fills half of the 32-wide matrix tiles: the library runs it at 32 on copies of the
                             tensors padded with zero features, kept in the workspace (which grows by those copies);
                             results are those of the 16-wide problem, the cost is that of head_dim 32 plus the copies */
       MTFM_HTA_FP32 = 1  /* float32 storage and arithmetic (plain FMA debug path); 1 <= head_dim <= 128 */ };

/* which layer of a block: queries = all tokens, or target tokens only */
enum { MTFM_HTA_LAYER_FULL = 0, MTFM_HTA_LAYER_TARGET = 1 };

/*
 * Bytes of device workspace a call with these sizes needs (0 is possible).  Pure host arithmetic.
 * The bf16 path keeps there what it builds on the device at the start of every call -- the work
 * counters of its persistent kernels and the user schedule (users ordered by decreasing number of
 * attention tiles, from hist_len / n_targets) -- and, for the backward pass, two float32 values per
 * (query head, query row): -delta = -<dout, out> and -lse / softmax_scale.
 * A forward call on so few users that (user, kv head, row tile) items cannot give every compute unit a workgroup
 * (a handful of requests at inference; decided from batch, the max_* bounds and the head shape alone) splits the keys
 * of each item over several workgroups; the workspace then also holds their partial results, float32
 * [splits][total_q][Hq][head_dim] and [splits][Hq][total_q], which a second kernel merges into out and lse.
 * is_bwd = 0 for mtfm_hta_fwd, 1 for mtfm_hta_bwd.  Returns (size_t)-1 for invalid arguments.
 * The workspace must be 256-byte aligned; its contents are undefined before and after a call and it
 * may be reused by the next call on the same stream.  Two calls that run at the same time (on
 * different streams) need a workspace each.
 */
MTFM_HTA_API size_t mtfm_hta_workspace_bytes(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q,
                                int64_t total_kv, int32_t max_hist, int32_t max_targets, int32_t Hq,
                                int32_t Hkv, int32_t head_dim);

/*
 * Forward: out = softmax_over_visible_keys(softmax_scale * Q K^T) V per user and head, and the
 * logsumexp of every query row (Eq. for A^(l,h) of the full layer, A_T^(l,h) of the target layer).
 *   q           in   [total_q][Hq][head_dim]
 *   k, v        in   [total_kv][Hkv][head_dim]
 *   out         out  [total_q][Hq][head_dim]   fully overwritten (bf16: rounded to nearest even)
 *   lse         out  [Hq][total_q] float32     fully overwritten
 *   q_offsets, kv_offsets  in  [batch+1] int32; hist_len, n_targets  in  [batch] int32 (all >= 0)
 *   total_q, total_kv      = q_offsets[batch], kv_offsets[batch] (host copies, < 2^31)
 *   max_hist, max_targets  host-known upper bounds of hist_len[] / n_targets[] (they size the launch)
 *   softmax_scale          > 0, finite; typically 1/sqrt(head_dim)
 * Data pointers must be 16-byte aligned.  batch == 0 or total_q == 0 is a successful no-op.
 * workspace: mtfm_hta_workspace_bytes(..., is_bwd = 0, ...) bytes, 256-byte aligned (none for fp32).
 */
MTFM_HTA_API int mtfm_hta_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
                 const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                 const int32_t* n_targets, int32_t batch, int64_t total_q, int64_t total_kv,
                 int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim,
                 float softmax_scale, int dtype, int layer, void* workspace, size_t workspace_bytes,
                 void* stream);

/*
 * mtfm_hta_fwd for callers that cannot allocate device memory or hand over a workspace: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as mtfm_hta_fwd
 * without `workspace` / `workspace_bytes`: what that call keeps in the caller's workspace (work counters, user
 * schedule, the partial results of a forward pass that splits its keys) lives in a buffer of
 * MTFM_HTA_STATIC_SCRATCH_BYTES built into the library, one copy in the memory of each GPU the library has run on,
 * held until the process ends.  The call allocates and frees nothing, on the host or on the device.
 * A call that needs more scratch memory than that (mtfm_hta_workspace_bytes(..., is_bwd = 0, ...) says how much; only
 * a forward pass that splits its keys over many partial results can, e.g. several requests with hundreds of
 * candidates at head_dim 128) returns MTFM_HTA_ERR_WORKSPACE and enqueues nothing; use mtfm_hta_fwd then.
 * All calls on one GPU share that GPU's buffer: calls that may overlap in time (different streams, different threads)
 * race and must be serialised by the caller, or use mtfm_hta_fwd with a workspace each.  Consecutive calls on one
 * stream are safe.  The buffer's address is looked up on the first call on each device; make that first call
 * outside a graph capture.
 */
#define MTFM_HTA_STATIC_SCRATCH_BYTES (8u << 20)
MTFM_HTA_API int mtfm_hta_fwd_static(const void* q, const void* k, const void* v, void* out, float* lse,
                 const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                 const int32_t* n_targets, int32_t batch, int64_t total_q, int64_t total_kv,
                 int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim,
                 float softmax_scale, int dtype, int layer, void* stream);

/*
 * Backward of mtfm_hta_fwd for an upstream gradient dout: the probabilities are recomputed from the
 * saved logsumexp, p_ij = exp(scale*s_ij - lse_i), then with delta_i = <dout_i, out_i>,
 * ds_ij = p_ij (<dout_i, v_j> - delta_i):
 *   dq_i = scale * sum_j ds_ij k_j,   dk_j = scale * sum_{h in group} sum_i ds_ij q_i,
 *   dv_j = sum_{h in group} sum_i p_ij dout_i        (gradient of the two attention equations above).
 *   dout, q, out  in  [total_q][Hq][head_dim];  k, v  in  [total_kv][Hkv][head_dim];  lse  in  [Hq][total_q]
 *   dq            out [total_q][Hq][head_dim]   fully overwritten
 *   dk, dv        out [total_kv][Hkv][head_dim] fully overwritten (in a target layer history rows receive the
 *                 gradient of every target query, target rows that of their own query)
 * `out` and `lse` must be what mtfm_hta_fwd produced for the same inputs.  Remaining arguments as in
 * mtfm_hta_fwd.  batch == 0 or total_kv == 0 is a successful no-op; with total_q == 0 (a target layer whose
 * users have no candidate) the row-shaped tensors are empty and may be null, and dk = dv = 0 is written.
 * The bf16 path needs a workspace (mtfm_hta_workspace_bytes with is_bwd = 1) and is bitwise reproducible;
 * the fp32 debug path sums dk/dv with float32 atomics, so it is reproducible to rounding only.
 */
MTFM_HTA_API int mtfm_hta_bwd(const void* dout, const void* q, const void* k, const void* v, const void* out,
                 const float* lse, void* dq, void* dk, void* dv, const int32_t* q_offsets,
                 const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* n_targets,
                 int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist,
                 int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float softmax_scale,
                 int dtype, int layer, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Host-side check of host copies of the jagged arrays (tests and callers that have them on the host):
 * monotone offsets, kv_offsets[b+1]-kv_offsets[b] == hist_len[b]+n_targets[b], the q_offsets rule of
 * `layer`, bounds respected.  All pointers are HOST pointers.  Returns MTFM_HTA_OK or
 * MTFM_HTA_ERR_INVALID_ARG (with mtfm_hta_last_error() naming the first violation).
 */
MTFM_HTA_API int mtfm_hta_validate_host(const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                           const int32_t* n_targets, int32_t batch, int64_t total_q, int64_t total_kv,
                           int32_t max_hist, int32_t max_targets, int layer);

/*
 * Samples with real-time tokens (mask rule 2 of the dynamic mask, Section 3.2.2: a real-time key may be attended to
 * only by queries whose timestamp is later than its own).  The K/V rows of user b are then hist_len[b] history tokens, rt_len[b] real-time
 * tokens, n_targets[b] target tokens, in this order (X = (H; R; T), Section 3.2.1); the queries of a full layer are
 * all of them, those of a target layer the target tokens.  Visibility of key j for query i:
 *   history key: always (rule 1);   target key: j == i (rule 3);
 *   real-time key: timestamps[j] < timestamps[i], or j == i (rule 2: later is strict, for every kind of query token;
 *   a real-time token sees itself, like a target token, so that no row is empty).
 * Additional arguments, otherwise exactly as the functions without the suffix (which are the case rt_len == 0):
 *   rt_len      in  [batch] int32 (>= 0)          device pointer
 *   timestamps  in  [total_kv] int32, one per K/V row; the real-time tokens of a user must be sorted by
 *               non-decreasing timestamp (history and target tokens in any order)        device pointer
 *   max_rt      host-known upper bound of rt_len[]
 *   kv_offsets  prefix sums of hist_len + rt_len + n_targets;  q_offsets == kv_offsets in a full layer
 * The workspace (mtfm_hta_workspace_bytes_rt) also holds one int32 per query row: the number of leading K/V rows of
 * its user (history, then the real-time tokens strictly earlier than the row) it attends to; the fp32 path needs
 * it as well.  mtfm_hta_validate_host_rt additionally checks the order of the real-time timestamps.
 */
MTFM_HTA_API size_t mtfm_hta_workspace_bytes_rt(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q,
                                int64_t total_kv, int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq,
                                int32_t Hkv, int32_t head_dim);
MTFM_HTA_API int mtfm_hta_fwd_rt(const void* q, const void* k, const void* v, void* out, float* lse,
                 const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* rt_len,
                 const int32_t* n_targets, const int32_t* timestamps, int32_t batch, int64_t total_q, int64_t total_kv,
                 int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim,
                 float softmax_scale, int dtype, int layer, void* workspace, size_t workspace_bytes, void* stream);
MTFM_HTA_API int mtfm_hta_bwd_rt(const void* dout, const void* q, const void* k, const void* v, const void* out,
                 const float* lse, void* dq, void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets,
                 const int32_t* hist_len, const int32_t* rt_len, const int32_t* n_targets, const int32_t* timestamps,
                 int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_rt,
                 int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float softmax_scale, int dtype,
                 int layer, void* workspace, size_t workspace_bytes, void* stream);
MTFM_HTA_API int mtfm_hta_validate_host_rt(const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                 const int32_t* rt_len, const int32_t* n_targets, const int32_t* timestamps, int32_t batch,
                 int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_rt, int32_t max_targets, int layer);

/* Message for the calling thread's most recent non-OK status ("" if none).  Points to thread-local
 * static storage owned by the library: do not free; valid until the thread's next failing call. */
MTFM_HTA_API const char* mtfm_hta_last_error(void);

/* Library version, "major.minor.patch"; static storage. */
MTFM_HTA_API const char* mtfm_hta_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MTFM_HTA_H */
