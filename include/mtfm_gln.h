/*
 * mtfm_gln.h -- C ABI of the fused Group Layer Normalization (GLN) of libmtfm_hta.so, hand-written for
 * AMD gfx950 (MI355X).
 *
 * The operation (Section 3.2.2: every token of a layer's input belongs to a group -- one per history sequence,
 * per real-time sequence, per scenario -- and is normalised with that group's parameters, X~ = GLN(X); the
 * attention result is normalised the same way and gated, GLN(A) (.) U, before the output map f2.  Section 3.3.2:
 * one fused operator does this in place of gathering each group's tokens, normalising them and scattering
 * them back):
 *   mean_i = (1/d) sum_c x_ic      var_i = (1/d) sum_c (x_ic - mean_i)^2      rstd_i = 1 / sqrt(var_i + eps)
 *   y_i    = (gamma[g_i] (.) (x_i - mean_i) rstd_i + beta[g_i])  [(.) u_i when a gate is given]
 * with g_i = group_id[i].  Readings fixed where the paper is silent: the statistics are per token over its
 * d_model features (a LayerNorm), what is grouped are the affine parameters; the variance is the biased one;
 * eps is an explicit argument.  Tokens are never moved: a token reads its group's parameter row where it lies.
 * Backward, for the upstream gradient dy of y (xhat_i = (x_i - mean_i) rstd_i):
 *   dz_i = dy_i (.) u_i (dy_i without a gate)        du_i = dy_i (.) (gamma[g_i] (.) xhat_i + beta[g_i])
 *   dgamma[g] = sum_{i in g} dz_i (.) xhat_i         dbeta[g] = sum_{i in g} dz_i
 *   w_i = dz_i (.) gamma[g_i]                        dx_i = rstd_i (w_i - mean_c(w_i) - xhat_i mean_c(w_i (.) xhat_i))
 *
 * Layout.  x, gate, y, dy, dx, dgate: [n_tokens][d_model] row-major, element type `dtype` (MTFM_HTA_BF16 or
 * MTFM_HTA_FP32), 16-byte aligned.  group_id: [n_tokens] int32 in [0, n_groups) (an id outside that range is
 * treated as the nearest valid one; mtfm_gln_validate_host() checks a host copy).  gamma, beta, dgamma, dbeta:
 * [n_groups][d_model] float32, 16-byte aligned.  mean, rstd: [n_tokens] float32.  All arithmetic is float32;
 * bf16 outputs are rounded to nearest even once, at the store.
 * Limits: d_model a positive multiple of 8, at most 2048; n_groups * roundup(d_model, 512) <= 8192 (the
 * parameter rows, and in the backward pass the gradient accumulators, live in the 160 KB of LDS).
 *
 * Pointers are DEVICE pointers owned by the caller unless stated otherwise; `stream` is a hipStream_t passed as
 * void* (NULL = the default stream).  The calls validate their scalar arguments on the host, enqueue kernels and
 * return; they never allocate, copy to the host or synchronise.  Status codes and mtfm_hta_last_error() are
 * those of mtfm_hta.h; on a non-zero status other than MTFM_HTA_ERR_LAUNCH nothing has been enqueued.
 */
#ifndef MTFM_GLN_H
#define MTFM_GLN_H

#include "mtfm_hta.h"

#ifdef __cplusplus
extern "C" {
#endif

/* kernel kinds of this header for mtfm_hta_timing_read() */
enum { MTFM_GLN_KERNEL_FWD = 4,        /* forward */
       MTFM_GLN_KERNEL_BWD = 5,        /* backward: dx, dgate and each workgroup's share of dgamma / dbeta */
       MTFM_GLN_KERNEL_BWD_REDUCE = 6  /* sum of the workgroups' shares */ };

/*
 * Forward.  `gate` may be NULL (plain GLN, the layer input of Section 3.2.2) or hold U (the gated output path).
 * `mean` and `rstd` receive the per-token statistics the backward pass reads; either may be NULL when no
 * backward pass follows.  y must not overlap x or gate.  n_tokens = 0 is valid, enqueues nothing and accepts
 * NULL arrays.
 */
MTFM_HTA_API int mtfm_gln_fwd(const void* x, const void* gate, const int32_t* group_id, const float* gamma,
                 const float* beta, void* y, float* mean, float* rstd, int64_t n_tokens, int32_t d_model,
                 int32_t n_groups, float eps, int dtype, void* stream);

/*
 * Bytes of device workspace mtfm_gln_bwd() needs (0 if the shape is invalid or unsupported): one float32 share
 * of dgamma and dbeta per workgroup of the backward kernel, whose grid has a fixed upper bound, so the size
 * depends on d_model and n_groups only.
 */
MTFM_HTA_API size_t mtfm_gln_bwd_workspace_bytes(int32_t d_model, int32_t n_groups);

/*
 * Backward.  mean, rstd are the forward pass's outputs for the same x.  gate and dgate are both NULL or both
 * given; beta is read only with a gate.  dx, dgate must not overlap the inputs.  dgamma and dbeta are overwritten
 * (rows of groups without tokens become zero; n_tokens = 0 zeroes both, and then the per-token arrays may be
 * NULL).  Their sums are formed in float32: within a workgroup with LDS atomic adds, whose order is not fixed, so
 * the last bits can differ from run to run; across workgroups in a fixed order.  `workspace`: 256-byte aligned, at least mtfm_gln_bwd_workspace_bytes();
 * contents need not be initialised and are not preserved.
 */
MTFM_HTA_API int mtfm_gln_bwd(const void* dy, const void* x, const void* gate, const int32_t* group_id,
                 const float* gamma, const float* beta, const float* mean, const float* rstd, void* dx, void* dgate,
                 float* dgamma, float* dbeta, int64_t n_tokens, int32_t d_model, int32_t n_groups, int dtype,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Checks a HOST copy of group_id: every id in [0, n_groups).  Returns MTFM_HTA_OK or MTFM_HTA_ERR_INVALID_ARG
 * (mtfm_hta_last_error() names the first offending token). */
MTFM_HTA_API int mtfm_gln_validate_host(const int32_t* group_id, int64_t n_tokens, int32_t n_groups);

#ifdef __cplusplus
}
#endif
#endif /* MTFM_GLN_H */
