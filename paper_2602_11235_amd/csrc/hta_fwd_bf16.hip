// bf16 forward kernel of Hybrid Target Attention for gfx950: QK^T and PV on the 32x32x16 bf16 MFMA
// with float32 accumulation, online softmax, K/V tiles staged in LDS once per key/value head and
// shared by the query heads of the GQA group (g = h / r, Section 3.2.2).
//
// Block skipping from the hybrid mask (rules 1 and 3): every query row of a user attends to all
// L_b history keys and never to another token's target key, so the only tiles ever issued are
// (row tile) x (history key tile); the single self key of a target row is added as one extra
// online-softmax step per row in the epilogue.  No mask is stored or loaded; only the ragged last
// history tile needs a bound check.
//
// Work decomposition: one workgroup = (user, kv head, chunk of `hpb` query heads of that group,
// tile of BM query rows).  Wave w serves head (w % hpb) of the chunk and the row group (w / hpb);
// it keeps RB blocks of 32 query rows in registers.  S is computed transposed, S^T = K Q^T, so
// a lane owns one query row: the row maximum and sum are reductions over the lane's own
// registers plus one exchange with the other half of the wave, and P^T in accumulator layout is
// directly the B operand of O^T = V^T P^T.  V stays row-major in LDS and is read through the LDS
// transpose read.
#include "../../include/mtfm_hta.h"
#include "../../include/mtfm_hta_timing.h"
#include "hta_common.h"
#include "hta_mfma.h"
#include "hta_tiles.h"

namespace hta {
namespace {

constexpr int BN = 64;  // keys per LDS tile
constexpr float RESCALE_SLACK = 8.f;  // log2 units a row's logits may exceed its softmax reference before a rescale

// What a wave of the row-stationary forward pass keeps in registers -- the Q fragments of its RB blocks of 32 query
// rows (one head), the running softmax state and the O^T accumulators -- and the steps on it.
//
// RT: the users carry real-time tokens (mask rule 2).  Their keys follow the history keys in the K/V rows and run through
// the same tile loop; a sub-tile that reaches past the history is masked per query row with the row's limit
// (p.lim: history + the real-time tokens strictly earlier than the row), and a real-time row gets its own key in the
// epilogue exactly like a target row.
//
// PW: the pointwise reading of phi2 -- weights norm * silu(scale s) on the same tiles and mask: no running maximum, no
// row sum, no lse; the accumulator holds sum_k s sigma(scale s) v and is scaled by norm * scale at the store.
template <int D, int RB, bool RT, bool PW>
struct FwdRows {
    static constexpr int NKS = D / 16, NDB = D / 32;
    bf16x8 qf[RB][NKS];  // B operand of S^T = K Q^T: lane = query row, 8 consecutive d values per k-step
    int lim[RB];         // leading keys the lane's row sees (RT; the history length otherwise)
    float m[RB], l[RB];
    floatx16 O[RB][NDB];
    // lane constants
    int nat[NKS], tlo[NDB], thi[NDB];  // element offsets of the operand fragments inside a swizzled tile
    int hf;
    float scale, c2, neg_c2;   // logits are handled in the log2 domain: c2 = scale log2(e)

    __device__ __forceinline__ void init_lane(const Params& p, int lane) {
        hf = lane >> 5;
        scale = p.scale;
        c2 = p.scale * LOG2E;
        neg_c2 = -c2;
        natural_offsets<D>(nat, lane);
        transposed_offsets<D>(tlo, thi, lane);
    }

    __device__ __forceinline__ void reset() {
#pragma unroll
        for (int rb = 0; rb < RB; rb++) {
            m[rb] = -INFINITY;
            l[rb] = 0.f;
#pragma unroll
            for (int db = 0; db < NDB; db++)
#pragma unroll
                for (int v = 0; v < 16; v++) O[rb][db][v] = 0.f;
        }
    }

    // Q fragments of rows wrow0 .. wrow0 + 32 RB - 1 of head h.  Rows past the end of the user are clamped to the last
    // row (n_rows >= 1); their results are never stored.
    __device__ __forceinline__ void load_q(const Params& p, int64_t q_base, int h, int wrow0, int n_rows, int L, int lane) {
        const int l32 = lane & 31, hf = lane >> 5;
        const __bf16* qg = (const __bf16*)p.q;
#pragma unroll
        for (int rb = 0; rb < RB; rb++) {
            int row = wrow0 + rb * 32 + l32;
            row = row < n_rows ? row : n_rows - 1;
            const __bf16* qp = qg + ((q_base + row) * p.Hq + h) * D + 8 * hf;
#pragma unroll
            for (int ks = 0; ks < NKS; ks++) qf[rb][ks] = *(const bf16x8*)(qp + ks * 16);
            lim[rb] = RT ? p.lim[q_base + row] : L;
        }
    }

    // One online-softmax step over a 32-key sub-tile that starts at key k0 (Ks, Vs: its first rows in LDS).  `n_live` =
    // number of keys of the sub-tile that exist (32 except in the ragged last tile), L = history length of the user.
    __device__ __forceinline__ void subtile(const __bf16* Ks, const __bf16* Vs, int n_live, int k0, int L) {
        const bool masked = RT && k0 + 32 > L;  // uniform: the sub-tile holds real-time keys (or runs past the end)
        if (masked) {
            bool any = false;
#pragma unroll
            for (int rb = 0; rb < RB; rb++) any = any || lim[rb] > k0;
            if (__builtin_amdgcn_ballot_w64(any) == 0) return;  // no row of this wave sees any key of the sub-tile
        }
        // S^T[key][row] = sum_d K[key][d] Q[row][d]
        floatx16 S[RB];
#pragma unroll
        for (int rb = 0; rb < RB; rb++)
#pragma unroll
            for (int v = 0; v < 16; v++) S[rb][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            const bf16x8 kf = *(const bf16x8*)(Ks + nat[ks]);
#pragma unroll
            for (int rb = 0; rb < RB; rb++) S[rb] = mfma32(kf, qf[rb][ks], S[rb]);
        }
        // Register v of the lane holds key 8 (v / 4) + 4 hf + v % 4 of the sub-tile; it is masked when that is >= the
        // number of visible keys, written as 4 hf - visible >= -(8 (v / 4) + v % 4): one subtraction per lane and
        // comparisons with constants, instead of sixteen lane constants kept in registers.
        if (masked) {  // per row: keys at or past the row's limit are not visible
            static_for<0, RB>([&](auto Rb) {
                constexpr int rb = decltype(Rb)::value;
                const int over = 4 * hf - (lim[rb] - k0);
                static_for<0, 16>([&](auto V) {
                    constexpr int v = decltype(V)::value;
                    S[rb][v] = (over >= -(8 * (v / 4) + (v % 4))) ? (PW ? PW_MASKED : -INFINITY) : S[rb][v];
                });
            });
        } else if (n_live < 32) {  // ragged: keys >= L_b are not visible
            const int over = 4 * hf - n_live;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                if (over >= -(8 * (v / 4) + (v % 4))) {
#pragma unroll
                    for (int rb = 0; rb < RB; rb++) S[rb][v] = PW ? PW_MASKED : -INFINITY;
                }
            }
        }
        bf16x8 pf[RB][2];
        if constexpr (PW) {
#pragma unroll
            for (int rb = 0; rb < RB; rb++)
#pragma unroll
                for (int v = 0; v < 16; v++)
                    pf[rb][v / 8][v % 8] = (__bf16)pw_silu(S[rb][v], pw_sigmoid(S[rb][v], neg_c2));  // s sigma(scale s): `scale` waits for the store
        } else {
            // Online softmax, one query row per lane (two lanes, 32 apart, share a row).  The reference m[rb]
            // of a row only has to bound its logits from above up to a modest factor: weights are exp2(s - m), sums
            // and outputs share the reference, and the final division by l removes it.  So the weights are formed
            // against the reference as it stands, without looking for the maximum first; the lane's sum of its 16
            // weights tells whether that was good enough: at most SUM_CAP = 16 * 2^RESCALE_SLACK when no logit exceeds
            // the reference by more than the slack (and inf or NaN while the reference is still -inf).  Only when some
            // lane of the wave fails that test -- in the first sub-tile of a row, and the handful of times a row
            // outgrows its reference -- is the maximum taken, the reference raised, the accumulators rescaled and
            // the weights formed again.  (The sum uses the rounded weights, the same as the P V product.)
            constexpr float SUM_CAP = 4096.f;
            static_assert(RESCALE_SLACK == 8.f, "SUM_CAP is 16 * 2^RESCALE_SLACK");
            static_for<0, RB>([&](auto Rb) {
                constexpr int rb = decltype(Rb)::value;
                auto weights = [&](float ref) __attribute__((always_inline)) {
#pragma unroll
                    for (int v = 0; v < 16; v++) pf[rb][v / 8][v % 8] = (__bf16)fast_exp2(fmaf(S[rb][v], c2, -ref));
                    float s0 = 0.f, s1 = 0.f;
                    add_bf16x8(s0, s1, pf[rb][0]);
                    add_bf16x8(s0, s1, pf[rb][1]);
                    return s0 + s1;
                };
                // (a row that has seen no key yet has the reference -inf: with real-time masks it may hold only masked
                // logits; keep -inf - -inf out)
                float lt = weights(RT ? fmaxf(m[rb], -1e30f) : m[rb]);
                if (__builtin_amdgcn_ballot_w64(!(lt <= SUM_CAP)) != 0) {
                    float mx = S[rb][0];
#pragma unroll
                    for (int v = 1; v < 16; v++) mx = fmaxf(mx, S[rb][v]);
                    mx = fmaxf(mx, other_half(mx)) * c2;
                    const bool grow = mx > m[rb] + RESCALE_SLACK;
                    const float m_new = grow ? mx : m[rb];
                    // 1 for the rows that keep their reference (which may still be -inf when rows see different keys)
                    const float alpha = grow ? fast_exp2(m[rb] - m_new) : 1.f;
                    m[rb] = m_new;
                    l[rb] *= alpha;
#pragma unroll
                    for (int db = 0; db < NDB; db++)
#pragma unroll
                        for (int v = 0; v < 16; v++) O[rb][db][v] *= alpha;
                    lt = weights(RT ? fmaxf(m_new, -1e30f) : m_new);
                }
                l[rb] += lt;
            });
        }
        // O^T[d][row] += sum_key V[key][d] P^T[key][row]
#pragma unroll
        for (int db = 0; db < NDB; db++)
#pragma unroll
            for (int s2 = 0; s2 < 2; s2++) {
                const bf16x8 vf = lds_read_tr_pair(Vs + 16 * s2 * D + tlo[db], Vs + 16 * s2 * D + thi[db]);
#pragma unroll
                for (int rb = 0; rb < RB; rb++) O[rb][db] = mfma32(vf, pf[rb][s2], O[rb][db]);
            }
    }

    // the 64-key tile at Ks / Vs whose first key is k0, of a user with LK keys in the tile loop and L history keys
    // the 64-key tile at Ks / Vs whose first key is k0, of a user with LK keys in the tile loop and L history keys
    __device__ __forceinline__ void tile(const __bf16* Ks, const __bf16* Vs, int k0, int LK, int L) {
#pragma unroll
        for (int kb = 0; kb < BN / 32; kb++) {
            const int n_live = LK - k0 - kb * 32;
            if (n_live > 0) subtile(Ks + kb * 32 * D, Vs + kb * 32 * D, n_live, k0 + kb * 32, L);
        }
    }

    // own key of target rows (rule 3) and of real-time rows: one more online-softmax step, straight from global memory
    __device__ __forceinline__ void own_key(const Params& p, int64_t kv_base, int g, int wrow0, int n_rows, int tok_shift, int L,
                                            int lane) {
        const int l32 = lane & 31, hf = lane >> 5;
        const __bf16* kg = (const __bf16*)p.k;
        const __bf16* vg = (const __bf16*)p.v;
#pragma unroll
        for (int rb = 0; rb < RB; rb++) {
            const int row = wrow0 + rb * 32 + l32;
            const int tok = tok_shift + row;
            if (row < n_rows && tok >= L) {
                const int64_t off = ((kv_base + tok) * p.Hkv + g) * D;
                const __bf16* kp = kg + off + 8 * hf;
                float dot = 0.f;
#pragma unroll
                for (int ks = 0; ks < NKS; ks++) {
                    const bf16x8 kk = *(const bf16x8*)(kp + ks * 16);
#pragma unroll
                    for (int j = 0; j < 8; j++) dot = fmaf((float)qf[rb][ks][j], (float)kk[j], dot);
                }
                dot += other_half(dot);
                float alpha = 1.f, ps;
                if constexpr (PW) {
                    ps = pw_silu(dot, pw_sigmoid(dot, neg_c2));
                } else {
                    const float s2 = dot * c2;
                    const float m_new = fmaxf(m[rb], s2);
                    alpha = fast_exp2(m[rb] - m_new);
                    ps = fast_exp2(s2 - m_new);
                    m[rb] = m_new;
                    l[rb] = l[rb] * alpha + (hf == 0 ? ps : 0.f);
                }
#pragma unroll
                for (int db = 0; db < NDB; db++)
#pragma unroll
                    for (int v4 = 0; v4 < 4; v4++) {
                        const bf16x4 vv = *(const bf16x4*)(vg + off + db * 32 + 8 * v4 + 4 * hf);
#pragma unroll
                        for (int j = 0; j < 4; j++) O[rb][db][4 * v4 + j] = fmaf(O[rb][db][4 * v4 + j], alpha, ps * (float)vv[j]);
                    }
            }
        }
    }

    // normalisation and stores.  SPLIT: the partial result of key split `split` -- rows normalised by their own sum
    // (0 when the split saw no key: lse = -inf), float32, with the logsumexp of its keys -- goes to the workspace.
    template <bool SPLIT>
    __device__ __forceinline__ void store(const Params& p, int64_t q_base, int h, int wrow0, int n_rows, int split, int lane) {
        const int l32 = lane & 31, hf = lane >> 5;
#pragma unroll
        for (int rb = 0; rb < RB; rb++) {
            const int row = wrow0 + rb * 32 + l32;
            const bool live = row < n_rows;
            const float lt = l[rb] + other_half(l[rb]);
            if (live && SPLIT) {
                const float inv = PW ? p.norm * scale : (lt > 0.f ? 1.f / lt : 0.f);
                float* op = p.o_part + (((int64_t)split * p.total_q + q_base + row) * p.Hq + h) * D;
#pragma unroll
                for (int db = 0; db < NDB; db++)
#pragma unroll
                    for (int v4 = 0; v4 < 4; v4++) {
                        floatx4 o4;
#pragma unroll
                        for (int j = 0; j < 4; j++) o4[j] = O[rb][db][4 * v4 + j] * inv;
                        *(floatx4*)(op + db * 32 + 8 * v4 + 4 * hf) = o4;
                    }
                if (!PW && hf == 0)
                    p.lse_part[((int64_t)split * p.Hq + h) * p.total_q + q_base + row] =
                        lt > 0.f ? (m[rb] + __builtin_amdgcn_logf(lt)) * LN2 : -INFINITY;
            } else if (live) {
                const float inv = PW ? p.norm * scale : 1.f / lt;
                __bf16* op = (__bf16*)p.out + ((q_base + row) * p.Hq + h) * D;
#pragma unroll
                for (int db = 0; db < NDB; db++)
#pragma unroll
                    for (int v4 = 0; v4 < 4; v4++) {
                        bf16x4 o4;
#pragma unroll
                        for (int j = 0; j < 4; j++) o4[j] = (__bf16)(O[rb][db][4 * v4 + j] * inv);
                        *(bf16x4*)(op + db * 32 + 8 * v4 + 4 * hf) = o4;
                    }
                if (!PW && hf == 0) p.lse[(int64_t)h * p.total_q + q_base + row] = (m[rb] + __builtin_amdgcn_logf(lt)) * LN2;
            }
        }
    }
};

// One workgroup per (user, kv head, chunk of query heads, tile of BM rows), from the launch grid.
//
// SPLIT: the launch has too few (user, kv head, row tile) items to fill the chip (a handful of requests at
// inference).  The grid gets a second dimension: workgroup (x, y) runs key tiles [y, y+1) * n_kt / n_splits of item x
// and leaves a partial result in the workspace; split 0 also takes the rows' own keys.  merge_splits_kernel combines
// the partial results (with PW they are plain partial sums, which it adds up).
template <int D, int RB, int NW, bool RT, bool SPLIT, bool PW = false>
__global__ __launch_bounds__(NW * 64, 2) void fwd_bf16_kernel(Params p, int hpb, int n_hc, int tpg) {
    using ST = KvStage<D, NW>;
    static_assert(ST::BN == BN, "tile height");
    // NSTAGE stages of [K tile][V tile], filled by asynchronous global -> LDS copies NSTAGE-1 tiles ahead of their use
    // (two ahead, except for d = 128 where a third stage would cost the second workgroup of the CU).  The compiler
    // never sees a store into this array (the copies are issued from inline assembly), so it neither orders LDS reads
    // against them nor drains them; the counted waits and barriers below do that.
    constexpr int NSTAGE = D <= 64 ? 3 : 2, AHEAD = NSTAGE - 1;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[NSTAGE * ST::BYTES];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const WorkItem w = decode_work(blockIdx.x, p.batch * p.Hkv * n_hc, p.Hkv * n_hc, tpg);
    if (!w.valid) return;
    const int b = scheduled_user(p, w.user_slot);
    const int g = w.y / n_hc, hc = w.y % n_hc;
    const int L = p.hist_len[b], T = p.n_targets[b];
    const int LK = L + (RT ? p.rt_len[b] : 0);  // keys that run through the tile loop: history, then real-time
    const int n_rows = p.layer == 0 ? LK + T : T;
    const int BM = (NW / hpb) * RB * 32;
    const int tile_row0 = w.tile * BM;
    if (tile_row0 >= n_rows) return;  // uniform for the whole workgroup
    const int r = p.Hq / p.Hkv;
    const int h = g * r + hc * hpb + wave % hpb;
    const int wrow0 = tile_row0 + (wave / hpb) * (RB * 32);
    const int tok_shift = p.layer == 0 ? 0 : LK;  // token index of query row 0
    const int64_t q_base = p.q_off[b], kv_base = p.kv_off[b];
    const __bf16* kg = (const __bf16*)p.k;
    const __bf16* vg = (const __bf16*)p.v;

    FwdRows<D, RB, RT, PW> rows;
    rows.init_lane(p, lane);
    rows.load_q(p, q_base, h, wrow0, n_rows, L, lane);
    rows.reset();

    const int n_kt_all = (LK + BN - 1) / BN;
    const int split = SPLIT ? (int)blockIdx.y : 0;
    const int t_lo = SPLIT ? split * n_kt_all / p.n_splits : 0;               // first key tile of this workgroup
    const int n_kt = (SPLIT ? (split + 1) * n_kt_all / p.n_splits : n_kt_all) - t_lo;  // and how many it runs
    uint32_t voff[ST::COPIES];
    ST::lane_offsets(voff, p.Hkv, wave, lane);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t smem_addr = lds_address(smem);

    // The first tiles are requested while the Q fragments are still on their way: one memory latency instead of two
    // at the start of every workgroup.  From the wait on, the only vector-memory traffic of the loop are the
    // asynchronous copies, which this code counts itself; the compiler must not be left with pending loads of its own
    // (the Q fragments) that it would wait for inside the loop.
    if (n_kt > 0) ST::issue(kg, vg, kv_base, p.Hkv, g, LK, t_lo, smem_addr, voff, wave_u, lane);
    if (AHEAD > 1 && n_kt > 1) ST::issue(kg, vg, kv_base, p.Hkv, g, LK, t_lo + 1, smem_addr + ST::BYTES, voff, wave_u, lane);
    wait_vmem_loads();
    lds_barrier();
    // (t counts from this workgroup's first tile.)  Tile t is consumed from stage t % NSTAGE while tile t+AHEAD is fetched into stage (t+AHEAD) % NSTAGE, which was
    // last read for tile t-1, i.e. before the barrier that every wave has passed.
    auto tile = [&](int t, auto St) __attribute__((always_inline)) {
        constexpr int st = decltype(St)::value;
        if (t + AHEAD < n_kt)
            ST::issue(kg, vg, kv_base, p.Hkv, g, LK, t_lo + t + AHEAD, smem_addr + ((st + AHEAD) % NSTAGE) * ST::BYTES, voff, wave_u, lane);
        const __bf16* Ks = (const __bf16*)(smem + st * ST::BYTES);
        rows.tile(Ks, Ks + ST::TILE, (t_lo + t) * BN, LK, L);
        // tile t+1 must have landed; a tile requested after it may stay in flight
        if (AHEAD > 1 && t + 2 < n_kt) wait_vmem_outstanding<ST::COPIES>(); else wait_vmem_outstanding<0>();
        lds_barrier();
    };
    for (int t = 0; t < n_kt; t += NSTAGE) {
        tile(t, std::integral_constant<int, 0>{});
        if (t + 1 < n_kt) tile(t + 1, std::integral_constant<int, 1>{});
        if constexpr (NSTAGE > 2) {
            if (t + 2 < n_kt) tile(t + 2, std::integral_constant<int, 2>{});
        }
    }

    if (split == 0) rows.own_key(p, kv_base, g, wrow0, n_rows, tok_shift, L, lane);
    rows.template store<SPLIT>(p, q_base, h, wrow0, n_rows, split, lane);
}

// out = sum_s w_s O_s / sum_s w_s with w_s = exp(lse_s - max lse), lse = max lse + log sum_s w_s: the exact
// combination of softmax results over disjoint key sets.  One thread per 4 features of a (row, head).
// PW: the partial results are partial sums of non-normalised weights: out = sum_s O_s, no lse.
template <bool PW>
__global__ __launch_bounds__(256) void merge_splits_kernel(Params p) {
    const int64_t quads = p.d / 4;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= p.total_q * p.Hq * quads) return;
    const int c = (int)(id % quads);
    const int64_t rh = id / quads;
    const int h = (int)(rh % p.Hq);
    const int64_t row = rh / p.Hq;
    // all loads of a thread are independent: issue them in batches of eight instead of one memory latency per split
    const float* lp = p.lse_part + (int64_t)h * p.total_q + row;
    const float* op = p.o_part + (row * p.Hq + h) * p.d + 4 * c;
    const int64_t l_stride = (int64_t)p.Hq * p.total_q, o_stride = p.total_q * p.Hq * p.d;
    float mx = -INFINITY;
    if constexpr (!PW) {
#pragma unroll 8
        for (int s = 0; s < p.n_splits; s++) mx = fmaxf(mx, lp[s * l_stride]);
    }
    float sum = 0.f;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int s = 0; s < p.n_splits; s++) {
        const float w = PW ? 1.f : __expf(lp[s * l_stride] - mx);
        const floatx4 o = *(const floatx4*)(op + s * o_stride);
        sum += w;
        acc += w * o;
    }
    const float inv = PW ? 1.f : 1.f / sum;
    bf16x4 o4;
#pragma unroll
    for (int j = 0; j < 4; j++) o4[j] = (__bf16)(acc[j] * inv);
    *(bf16x4*)((__bf16*)p.out + (row * p.Hq + h) * p.d + 4 * c) = o4;
    if (!PW && c == 0) p.lse[(int64_t)h * p.total_q + row] = mx + __logf(sum);
}

int gcd(int a, int b) { return b == 0 ? a : gcd(b, a % b); }

// launch geometry of the <D, RB, NW> kernel for a call's host-known bounds
struct Geometry {
    int hpb, n_hc;
    int64_t n_rt, n_items;  // row tiles per (user, kv head, head chunk) group; groups x row tiles
};
Geometry geometry_of(int RB, int NW, int32_t batch, int32_t Hq, int32_t Hkv, int64_t max_rows) {
    Geometry g;
    const int r = Hq / Hkv;
    g.hpb = gcd(r, NW);
    g.n_hc = r / g.hpb;
    const int BM = (NW / g.hpb) * RB * 32;
    g.n_rt = (max_rows + BM - 1) / BM;
    g.n_items = (int64_t)batch * Hkv * g.n_hc * g.n_rt;
    return g;
}

template <int D, int RB, int NW>
hipError_t launch(const Params& p, hipStream_t s) {
    const bool split = p.n_splits > 1;
    void (*kernel)(Params, int, int, int);
    if (p.pointwise) {
        kernel = p.rt_len ? (split ? fwd_bf16_kernel<D, RB, NW, true, true, true> : fwd_bf16_kernel<D, RB, NW, true, false, true>)
                          : (split ? fwd_bf16_kernel<D, RB, NW, false, true, true> : fwd_bf16_kernel<D, RB, NW, false, false, true>);
    } else {
        kernel = p.rt_len ? (split ? fwd_bf16_kernel<D, RB, NW, true, true> : fwd_bf16_kernel<D, RB, NW, true, false>)
                          : (split ? fwd_bf16_kernel<D, RB, NW, false, true> : fwd_bf16_kernel<D, RB, NW, false, false>);
    }
    const int64_t rows = max_query_rows(p);
    if (rows <= 0) return hipSuccess;
    const Geometry g = geometry_of(RB, NW, p.batch, p.Hq, p.Hkv, rows);
    const int64_t n_blocks = work_grid((int64_t)p.batch * p.Hkv * g.n_hc, g.n_rt);
    if (n_blocks >= (1ll << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)n_blocks, split ? p.n_splits : 1), dim3(NW * 64), 0, s, p, g.hpb, g.n_hc,
                       (int)g.n_rt);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && split) {
        const int64_t threads = p.total_q * p.Hq * (p.d / 4);
        if (p.pointwise)
            hipLaunchKernelGGL(merge_splits_kernel<true>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, p);
        else
            hipLaunchKernelGGL(merge_splits_kernel<false>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, p);
        e = hipGetLastError();
    }
    return e;
}

// (RB, NW) of the forward kernel for a head shape: eight waves of one 32-row block each whenever the head group fills
// them (r a multiple of 4) -- the small register footprint lets four waves share a SIMD, which hides more latency than
// a second row block per wave saves in LDS reads -- otherwise four waves with two row blocks each.
void kernel_shape(int32_t d, int32_t Hq, int32_t Hkv, int& RB, int& NW) {
    const bool wide = ((Hq / Hkv) % 4) == 0;
    NW = wide ? 8 : 4;
    RB = d == 32 ? 2 : (d == 64 ? (wide ? 1 : 2) : 1);
}

}  // namespace

bool bf16_supported(int32_t d, int32_t Hq, int32_t Hkv) {
    (void)Hq;
    (void)Hkv;
    return d == 32 || d == 64 || d == 128;
}

// Key splits of the forward pass: 1 (none) when the (user, kv head, row tile) items already give every compute unit
// a workgroup; otherwise enough splits for one workgroup per compute unit, each keeping at least MIN_TILES key tiles
// (measured on 1..8 requests with 2k..8k histories: two workgroups per unit or shorter splits only add partial
// results for the merge to read; fewer splits leave units idle).
int fwd_key_splits(int32_t batch, int32_t Hq, int32_t Hkv, int32_t d, int64_t max_rows, int64_t max_keys) {
    constexpr int64_t CUS = 256, MIN_TILES = 4, MAX_SPLITS = 32;
    if (batch <= 0 || max_rows <= 0 || !bf16_supported(d, Hq, Hkv)) return 1;
    int RB, NW;
    kernel_shape(d, Hq, Hkv, RB, NW);
    const Geometry g = geometry_of(RB, NW, batch, Hq, Hkv, max_rows);
    if (g.n_items >= CUS) return 1;
    const int64_t want = (CUS + g.n_items - 1) / g.n_items;
    const int64_t by_len = ((max_keys + BN - 1) / BN) / MIN_TILES;
    int64_t n = want < by_len ? want : by_len;
    n = n < MAX_SPLITS ? n : MAX_SPLITS;
    return n > 1 ? (int)n : 1;
}

hipError_t launch_fwd_bf16(const Params& p, hipStream_t s) {
    int RB, NW;
    kernel_shape(p.d, p.Hq, p.Hkv, RB, NW);
    const bool wide = NW == 8;
    hipError_t e;
    timing_begin(MTFM_HTA_KERNEL_FWD, s);
    switch (p.d) {
        case 32: e = wide ? launch<32, 2, 8>(p, s) : launch<32, 2, 4>(p, s); break;
        case 64: e = wide ? launch<64, 1, 8>(p, s) : launch<64, 2, 4>(p, s); break;
        case 128: e = wide ? launch<128, 1, 8>(p, s) : launch<128, 1, 4>(p, s); break;
        default: e = hipErrorInvalidValue;
    }
    timing_end(MTFM_HTA_KERNEL_FWD, s);
    return e;
}

}  // namespace hta
