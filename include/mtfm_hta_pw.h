/*
 * mtfm_hta_pw.h -- C ABI of the pointwise variant of Hybrid Target Attention in libmtfm_hta.so (AMD gfx950).
 *
 * Section 3.2.2 writes the attention of a layer as phi2(Q K^T (.) M) V and says only that phi2 is a nonlinearity,
 * while the layers are introduced as HSTU layers, whose attention weights are a pointwise SiLU that is not
 * normalised over the keys.  mtfm_hta.h takes the softmax reading; this header is the other one:
 *   out_i = norm * sum_{j visible to i} silu(scale <q_i, k_j>) v_j,      silu(x) = x / (1 + exp(-x)),
 * with the same dynamic mask (rules 1 and 3: history keys visible to every query, a target key only to itself),
 * grouped-query heads, full and target layers, data layout, pointer, stream and error conventions as mtfm_hta.h.
 * `scale` multiplies the dot products, `norm` the weights (HSTU divides by the sequence length: pass its
 * reciprocal); both must be positive and finite.  There are no row statistics: no lse is produced, and the backward
 * pass needs neither the forward output nor anything saved by the forward pass.  Backward, with x_ij = scale <q_i, k_j>:
 *   dv_j = norm sum_i silu(x_ij) dout_i        dx_ij = norm <dout_i, v_j> silu'(x_ij),  silu'(x) = s (1 + x (1 - s)), s = sigmoid(x)
 *   dq_i = scale sum_j dx_ij k_j               dk_j = scale sum_i dx_ij q_i             (sums over the query heads of a kv head)
 * bf16 with head_dim in {16, 32, 64, 128} on the MFMA kernels, fp32 on the debug path, as in mtfm_hta.h.  The functions
 * with the _rt suffix take samples with real-time tokens (mask rule 2), with the arguments and the readings of the
 * _rt functions of mtfm_hta.h.  A forward call on a few users splits the keys over workgroups as mtfm_hta_fwd does
 * (the partial results are partial sums here); the workspace functions account for it.
 */
#ifndef MTFM_HTA_PW_H
#define MTFM_HTA_PW_H

#include "mtfm_hta.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of device workspace a call needs (pure host arithmetic; (size_t)-1 for invalid arguments): the schedule
 * region of mtfm_hta.h, the partial results of a forward call that splits its keys, and, for the bf16 backward
 * pass, two float32 values per (query head, query row). */
MTFM_HTA_API size_t mtfm_hta_pw_workspace_bytes(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q,
                                int64_t total_kv, int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv,
                                int32_t head_dim);

/* Forward: `out` [total_q][Hq][head_dim] is fully overwritten.  Arguments as mtfm_hta_fwd, without lse. */
MTFM_HTA_API int mtfm_hta_pw_fwd(const void* q, const void* k, const void* v, void* out, const int32_t* q_offsets,
                 const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* n_targets, int32_t batch,
                 int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv,
                 int32_t head_dim, float scale, float norm, int dtype, int layer, void* workspace,
                 size_t workspace_bytes, void* stream);

/* Backward: dq [total_q][Hq][head_dim], dk, dv [total_kv][Hkv][head_dim] are fully overwritten (rows of tokens no
 * query sees become zero).  Arguments as mtfm_hta_bwd, without out and lse. */
MTFM_HTA_API int mtfm_hta_pw_bwd(const void* dout, const void* q, const void* k, const void* v, void* dq, void* dk,
                 void* dv, const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                 const int32_t* n_targets, int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist,
                 int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float scale, float norm, int dtype,
                 int layer, void* workspace, size_t workspace_bytes, void* stream);

/* Samples with real-time tokens: rt_len [batch] and timestamps [total_kv] (int32, device) and the bound max_rt are
 * extra, as in mtfm_hta_fwd_rt / mtfm_hta_bwd_rt; the workspace also holds one int32 per query row. */
MTFM_HTA_API size_t mtfm_hta_pw_workspace_bytes_rt(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q,
                                int64_t total_kv, int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq,
                                int32_t Hkv, int32_t head_dim);
MTFM_HTA_API int mtfm_hta_pw_fwd_rt(const void* q, const void* k, const void* v, void* out, const int32_t* q_offsets,
                 const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* rt_len, const int32_t* n_targets,
                 const int32_t* timestamps, int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist,
                 int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float scale, float norm,
                 int dtype, int layer, void* workspace, size_t workspace_bytes, void* stream);
MTFM_HTA_API int mtfm_hta_pw_bwd_rt(const void* dout, const void* q, const void* k, const void* v, void* dq, void* dk,
                 void* dv, const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                 const int32_t* rt_len, const int32_t* n_targets, const int32_t* timestamps, int32_t batch,
                 int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq,
                 int32_t Hkv, int32_t head_dim, float scale, float norm, int dtype, int layer, void* workspace,
                 size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MTFM_HTA_PW_H */
