/*
 * CPU oracle for Hybrid Target Attention (HTA) with grouped-query heads.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the GPU library and is never part of the product path.  It shares no code
 * with the HIP kernels and is deliberately plain: float64 throughout, one loop per index, the
 * mask evaluated per (query token, key token) from the token types, no tiling, no online
 * softmax, no skipping.
 *
 * What it computes (Section 3.2.2):
 *   full attention layer    A^(h)   = phi2(Q^(h)   K^(g)T (.) M  ) V^(g)     every token is a query
 *   target attention layer  A_T^(h) = phi2(Q_T^(h) K^(g)T (.) M_T) V^(g)     queries = T-tokens only,
 *                           M_T = the T-token rows of M, K/V from all tokens
 *   g = ceil(h / r) for 1-based h, r = H / G (grouped-query attention): with 0-based heads, g = h / r.
 *   Dynamic mask M: rule 1, history tokens are visible to every token; rule 2, a real-time token is
 *   visible only to tokens with later timestamps; rule 3, a target token is visible only to itself.
 *   The functions without the _rt suffix are the case without real-time tokens (rules 1 and 3).
 *
 * Readings where the paper is silent (kept identical in the GPU library):
 *   - phi2 is a row softmax over the visible keys; masked keys are excluded (weight exactly 0).
 *   - "X visible to Y" means query Y may attend to key X; rows of M are queries.
 *   - logits are scaled by an explicit softmax_scale argument.
 *   - lse is the natural-log logsumexp of the scaled visible logits.
 *   - rule 2: "later" is strict (key timestamp < query timestamp), for every kind of query token; in
 *     addition a real-time token sees itself, like a target token does, so that no row is empty.
 *
 *
 * The other reading of phi2 (the layers are described as HSTU layers, whose attention weights are a pointwise,
 * non-normalised nonlinearity): the hta_oracle_pw_* functions at the end of this file compute
 *   out_i = norm * sum_{j visible to i} silu(scale <q_i, k_j>) v_j,   silu(x) = x / (1 + exp(-x)),
 * with the same mask, heads and layers, and an explicit scalar `norm` (HSTU divides by the sequence length: the
 * caller passes its reciprocal).  No row statistics exist in this reading.
 *
 * Layout: q/out/dout/dq are [total_q][Hq][d]; k/v/dk/dv are [total_kv][Hkv][d]; lse is [Hq][total_q].
 * Per user b the K/V rows are L_b history tokens, then R_b real-time tokens, then T_b target tokens
 * (X = (H; R; T), Section 3.2.1), starting at kv_start[b]; ts[] holds one timestamp per K/V row.
 * Query rows start at q_start[b]: N_b = L_b + R_b + T_b rows in a full layer, T_b rows in a target layer.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { TOKEN_HISTORY = 0, TOKEN_REALTIME = 1, TOKEN_TARGET = 2 };
enum { LAYER_FULL = 0, LAYER_TARGET = 1 };

/* one user's sample: segment lengths and the timestamps of its tokens (NULL when it has no real-time tokens) */
typedef struct {
    int64_t hist_len, rt_len, n_targets;
    const int32_t* ts;
} sample_t;

/* type of token number `tok` (0-based within the user's sample) */
static int token_type(int64_t tok, const sample_t* u) {
    if (tok < u->hist_len) return TOKEN_HISTORY;
    if (tok < u->hist_len + u->rt_len) return TOKEN_REALTIME;
    return TOKEN_TARGET;
}

/* dynamic mask entry M[query token][key token] */
static int visible(int64_t query_tok, int64_t key_tok, const sample_t* u) {
    switch (token_type(key_tok, u)) {
        case TOKEN_HISTORY: return 1;                                                               /* rule 1 */
        case TOKEN_REALTIME: return u->ts[key_tok] < u->ts[query_tok] || key_tok == query_tok;      /* rule 2 */
        default: return key_tok == query_tok;                                                       /* rule 3 */
    }
}

static sample_t sample_of(int b, const int32_t* kv_start, const int32_t* hist_len, const int32_t* rt_len,
                          const int32_t* n_targets, const int32_t* ts) {
    sample_t u;
    u.hist_len = hist_len[b];
    u.rt_len = rt_len ? rt_len[b] : 0;
    u.n_targets = n_targets[b];
    u.ts = ts ? ts + kv_start[b] : NULL;
    return u;
}

int hta_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Forward.  rt_len and ts may both be NULL (no real-time tokens).  Returns 0, or -1 on bad scalar arguments. */
int hta_oracle_fwd_rt(const double* q, const double* k, const double* v, double* out, double* lse,
                      const int32_t* q_start, const int32_t* kv_start, const int32_t* hist_len,
                      const int32_t* rt_len, const int32_t* n_targets, const int32_t* ts, int32_t batch,
                      int64_t total_q, int32_t Hq, int32_t Hkv, int32_t d, double scale, int32_t layer) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || batch < 0) return -1;
    if (layer != LAYER_FULL && layer != LAYER_TARGET) return -1;
    if (rt_len && !ts) return -1;
    const int r = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < batch; b++) {
        for (int h = 0; h < Hq; h++) {
            const int g = h / r;
            const sample_t u = sample_of(b, kv_start, hist_len, rt_len, n_targets, ts);
            const int64_t N = u.hist_len + u.rt_len + u.n_targets;
            const int64_t first_tok = (layer == LAYER_FULL) ? 0 : u.hist_len + u.rt_len; /* token of query row 0 */
            const int64_t n_rows = N - first_tok;
            double* s = (double*)malloc((size_t)(N > 0 ? N : 1) * sizeof(double));
            for (int64_t row = 0; row < n_rows; row++) {
                const int64_t i = first_tok + row; /* query token */
                const double* qi = q + ((int64_t)(q_start[b] + row) * Hq + h) * d;
                double smax = -INFINITY;
                for (int64_t j = 0; j < N; j++) {
                    if (!visible(i, j, &u)) continue;
                    const double* kj = k + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                    double dot = 0.0;
                    for (int c = 0; c < d; c++) dot += qi[c] * kj[c];
                    s[j] = scale * dot;
                    if (s[j] > smax) smax = s[j];
                }
                double denom = 0.0;
                for (int64_t j = 0; j < N; j++)
                    if (visible(i, j, &u)) denom += exp(s[j] - smax);
                const double lse_i = smax + log(denom);
                double* oi = out + ((int64_t)(q_start[b] + row) * Hq + h) * d;
                for (int c = 0; c < d; c++) oi[c] = 0.0;
                for (int64_t j = 0; j < N; j++) {
                    if (!visible(i, j, &u)) continue;
                    const double p = exp(s[j] - lse_i);
                    const double* vj = v + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                    for (int c = 0; c < d; c++) oi[c] += p * vj[c];
                }
                lse[(int64_t)h * total_q + q_start[b] + row] = lse_i;
            }
            free(s);
        }
    }
    return 0;
}

/*
 * Backward of the forward above for an upstream gradient dout (softmax Jacobian written out):
 *   p_ij  = exp(s_ij - lse_i)            delta_i = <dout_i, out_i>
 *   dp_ij = <dout_i, v_j>                ds_ij   = p_ij (dp_ij - delta_i)
 *   dq_i  = scale sum_j ds_ij k_j        dk_j = scale sum_{h in g} sum_i ds_ij q_i
 *   dv_j  = sum_{h in g} sum_i p_ij dout_i
 * dq, dk, dv are fully overwritten.  `out` and `lse` must come from hta_oracle_fwd on the same inputs.
 */
int hta_oracle_bwd_rt(const double* dout, const double* q, const double* k, const double* v,
                      const double* out, const double* lse, double* dq, double* dk, double* dv,
                      const int32_t* q_start, const int32_t* kv_start, const int32_t* hist_len,
                      const int32_t* rt_len, const int32_t* n_targets, const int32_t* ts, int32_t batch,
                      int64_t total_q, int32_t Hq, int32_t Hkv, int32_t d, double scale, int32_t layer) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || batch < 0) return -1;
    if (layer != LAYER_FULL && layer != LAYER_TARGET) return -1;
    if (rt_len && !ts) return -1;
    const int r = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < batch; b++) {
        for (int g = 0; g < Hkv; g++) { /* one thread owns all of dk/dv[b, :, g, :] */
            const sample_t u = sample_of(b, kv_start, hist_len, rt_len, n_targets, ts);
            const int64_t N = u.hist_len + u.rt_len + u.n_targets;
            const int64_t first_tok = (layer == LAYER_FULL) ? 0 : u.hist_len + u.rt_len;
            const int64_t n_rows = N - first_tok;
            for (int64_t j = 0; j < N; j++) {
                double* dkj = dk + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                double* dvj = dv + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                for (int c = 0; c < d; c++) dkj[c] = dvj[c] = 0.0;
            }
            for (int h = g * r; h < (g + 1) * r; h++) {
                for (int64_t row = 0; row < n_rows; row++) {
                    const int64_t i = first_tok + row;
                    const int64_t qrow = (int64_t)(q_start[b] + row) * Hq + h;
                    const double* qi = q + qrow * d;
                    const double* doi = dout + qrow * d;
                    const double* oi = out + qrow * d;
                    double* dqi = dq + qrow * d;
                    const double lse_i = lse[(int64_t)h * total_q + q_start[b] + row];
                    double delta = 0.0;
                    for (int c = 0; c < d; c++) delta += doi[c] * oi[c];
                    for (int c = 0; c < d; c++) dqi[c] = 0.0;
                    for (int64_t j = 0; j < N; j++) {
                        if (!visible(i, j, &u)) continue;
                        const int64_t kvrow = (int64_t)(kv_start[b] + j) * Hkv + g;
                        const double* kj = k + kvrow * d;
                        const double* vj = v + kvrow * d;
                        double dot = 0.0, dp = 0.0;
                        for (int c = 0; c < d; c++) { dot += qi[c] * kj[c]; dp += doi[c] * vj[c]; }
                        const double p = exp(scale * dot - lse_i);
                        const double ds = p * (dp - delta);
                        double* dkj = dk + kvrow * d;
                        double* dvj = dv + kvrow * d;
                        for (int c = 0; c < d; c++) {
                            dqi[c] += scale * ds * kj[c];
                            dkj[c] += scale * ds * qi[c];
                            dvj[c] += p * doi[c];
                        }
                    }
                }
            }
        }
    }
    return 0;
}

/* Attention probabilities of one (user, head) as a dense [n_rows][N] matrix (0 where masked):
 * lets tests check that rows sum to one and inspect which pairs carry weight. */
int hta_oracle_probs_rt(const double* q, const double* k, double* probs, int32_t q_start, int32_t kv_start,
                        int32_t hist_len, int32_t rt_len, int32_t n_targets, const int32_t* ts, int32_t head,
                        int32_t Hq, int32_t Hkv, int32_t d, double scale, int32_t layer) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || head < 0 || head >= Hq) return -1;
    if (rt_len > 0 && !ts) return -1;
    const int r = Hq / Hkv, g = head / r;
    sample_t u;
    u.hist_len = hist_len;
    u.rt_len = rt_len;
    u.n_targets = n_targets;
    u.ts = ts ? ts + kv_start : NULL;
    const int64_t N = (int64_t)hist_len + rt_len + n_targets;
    const int64_t first_tok = (layer == LAYER_FULL) ? 0 : (int64_t)hist_len + rt_len;
    for (int64_t row = 0; row < N - first_tok; row++) {
        const int64_t i = first_tok + row;
        const double* qi = q + ((int64_t)(q_start + row) * Hq + head) * d;
        double* pr = probs + row * N;
        double smax = -INFINITY;
        for (int64_t j = 0; j < N; j++) {
            pr[j] = 0.0;
            if (!visible(i, j, &u)) continue;
            const double* kj = k + ((int64_t)(kv_start + j) * Hkv + g) * d;
            double dot = 0.0;
            for (int c = 0; c < d; c++) dot += qi[c] * kj[c];
            pr[j] = scale * dot;
            if (pr[j] > smax) smax = pr[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < N; j++)
            if (visible(i, j, &u)) denom += exp(pr[j] - smax);
        for (int64_t j = 0; j < N; j++) pr[j] = visible(i, j, &u) ? exp(pr[j] - smax) / denom : 0.0;
    }
    return 0;
}

/* The case without real-time tokens: every sample is history tokens followed by target tokens (rules 1 and 3). */
int hta_oracle_fwd(const double* q, const double* k, const double* v, double* out, double* lse,
                   const int32_t* q_start, const int32_t* kv_start, const int32_t* hist_len,
                   const int32_t* n_targets, int32_t batch, int64_t total_q, int32_t Hq, int32_t Hkv,
                   int32_t d, double scale, int32_t layer) {
    return hta_oracle_fwd_rt(q, k, v, out, lse, q_start, kv_start, hist_len, NULL, n_targets, NULL, batch, total_q, Hq,
                             Hkv, d, scale, layer);
}

int hta_oracle_bwd(const double* dout, const double* q, const double* k, const double* v,
                   const double* out, const double* lse, double* dq, double* dk, double* dv,
                   const int32_t* q_start, const int32_t* kv_start, const int32_t* hist_len,
                   const int32_t* n_targets, int32_t batch, int64_t total_q, int32_t Hq, int32_t Hkv,
                   int32_t d, double scale, int32_t layer) {
    return hta_oracle_bwd_rt(dout, q, k, v, out, lse, dq, dk, dv, q_start, kv_start, hist_len, NULL, n_targets, NULL,
                             batch, total_q, Hq, Hkv, d, scale, layer);
}

int hta_oracle_probs(const double* q, const double* k, double* probs, int32_t q_start, int32_t kv_start,
                     int32_t hist_len, int32_t n_targets, int32_t head, int32_t Hq, int32_t Hkv, int32_t d,
                     double scale, int32_t layer) {
    return hta_oracle_probs_rt(q, k, probs, q_start, kv_start, hist_len, 0, n_targets, NULL, head, Hq, Hkv, d, scale,
                               layer);
}


/* ---------------------------------------------------------------------------------------------------------------
 * Pointwise reading of phi2: out_i = norm * sum_{j visible to i} silu(scale <q_i, k_j>) v_j.
 * rt_len and ts may both be NULL.  Returns 0, or -1 on bad scalar arguments. */
static double silu(double x) { return x / (1.0 + exp(-x)); }
/* d silu / dx = sigma (1 + x (1 - sigma)) */
static double silu_prime(double x) {
    const double sg = 1.0 / (1.0 + exp(-x));
    return sg * (1.0 + x * (1.0 - sg));
}

int hta_oracle_pw_fwd_rt(const double* q, const double* k, const double* v, double* out, const int32_t* q_start,
                         const int32_t* kv_start, const int32_t* hist_len, const int32_t* rt_len,
                         const int32_t* n_targets, const int32_t* ts, int32_t batch, int32_t Hq, int32_t Hkv, int32_t d,
                         double scale, double norm, int32_t layer) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || batch < 0) return -1;
    if (layer != LAYER_FULL && layer != LAYER_TARGET) return -1;
    if (rt_len && !ts) return -1;
    const int r = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < batch; b++) {
        for (int h = 0; h < Hq; h++) {
            const int g = h / r;
            const sample_t u = sample_of(b, kv_start, hist_len, rt_len, n_targets, ts);
            const int64_t N = u.hist_len + u.rt_len + u.n_targets;
            const int64_t first_tok = (layer == LAYER_FULL) ? 0 : u.hist_len + u.rt_len;
            for (int64_t row = 0; row < N - first_tok; row++) {
                const int64_t i = first_tok + row;
                const double* qi = q + ((int64_t)(q_start[b] + row) * Hq + h) * d;
                double* oi = out + ((int64_t)(q_start[b] + row) * Hq + h) * d;
                for (int c = 0; c < d; c++) oi[c] = 0.0;
                for (int64_t j = 0; j < N; j++) {
                    if (!visible(i, j, &u)) continue;
                    const double* kj = k + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                    const double* vj = v + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                    double dot = 0.0;
                    for (int c = 0; c < d; c++) dot += qi[c] * kj[c];
                    const double a = norm * silu(scale * dot);
                    for (int c = 0; c < d; c++) oi[c] += a * vj[c];
                }
            }
        }
    }
    return 0;
}

/*
 * Backward of the pointwise forward:  x_ij = scale <q_i, k_j>,  a_ij = norm silu(x_ij)
 *   dv_j = sum_{h in g} sum_i a_ij dout_i            da_ij = <dout_i, v_j>
 *   dx_ij = norm da_ij silu'(x_ij)                   dq_i = scale sum_j dx_ij k_j     dk_j = scale sum_{h in g} sum_i dx_ij q_i
 */
int hta_oracle_pw_bwd_rt(const double* dout, const double* q, const double* k, const double* v, double* dq, double* dk,
                         double* dv, const int32_t* q_start, const int32_t* kv_start, const int32_t* hist_len,
                         const int32_t* rt_len, const int32_t* n_targets, const int32_t* ts, int32_t batch, int32_t Hq,
                         int32_t Hkv, int32_t d, double scale, double norm, int32_t layer) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || batch < 0) return -1;
    if (layer != LAYER_FULL && layer != LAYER_TARGET) return -1;
    if (rt_len && !ts) return -1;
    const int r = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < batch; b++) {
        for (int g = 0; g < Hkv; g++) { /* one thread owns all of dk/dv[b, :, g, :] */
            const sample_t u = sample_of(b, kv_start, hist_len, rt_len, n_targets, ts);
            const int64_t N = u.hist_len + u.rt_len + u.n_targets;
            const int64_t first_tok = (layer == LAYER_FULL) ? 0 : u.hist_len + u.rt_len;
            for (int64_t j = 0; j < N; j++) {
                double* dkj = dk + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                double* dvj = dv + ((int64_t)(kv_start[b] + j) * Hkv + g) * d;
                for (int c = 0; c < d; c++) dkj[c] = dvj[c] = 0.0;
            }
            for (int h = g * r; h < (g + 1) * r; h++) {
                for (int64_t row = 0; row < N - first_tok; row++) {
                    const int64_t i = first_tok + row;
                    const int64_t qrow = (int64_t)(q_start[b] + row) * Hq + h;
                    const double* qi = q + qrow * d;
                    const double* doi = dout + qrow * d;
                    double* dqi = dq + qrow * d;
                    for (int c = 0; c < d; c++) dqi[c] = 0.0;
                    for (int64_t j = 0; j < N; j++) {
                        if (!visible(i, j, &u)) continue;
                        const int64_t kvrow = (int64_t)(kv_start[b] + j) * Hkv + g;
                        const double* kj = k + kvrow * d;
                        const double* vj = v + kvrow * d;
                        double dot = 0.0, da = 0.0;
                        for (int c = 0; c < d; c++) { dot += qi[c] * kj[c]; da += doi[c] * vj[c]; }
                        const double x = scale * dot;
                        const double a = norm * silu(x);
                        const double dx = norm * da * silu_prime(x);
                        double* dkj = dk + kvrow * d;
                        double* dvj = dv + kvrow * d;
                        for (int c = 0; c < d; c++) {
                            dqi[c] += scale * dx * kj[c];
                            dkj[c] += scale * dx * qi[c];
                            dvj[c] += a * doi[c];
                        }
                    }
                }
            }
        }
    }
    return 0;
}
