// bf16 backward kernels of Hybrid Target Attention for gfx950.
//
// Gradient of A = softmax_visible(scale Q K^T) V (the two attention equations of Section 3.2.2)
// with the probabilities recomputed from the saved logsumexp:
//   P = exp(scale S - lse),  dP = dO V^T,  dS = P o (dP - delta),  delta_i = <dO_i, O_i>
//   dV = P^T dO,  dK = scale dS^T Q  (both summed over the query heads of the kv group),  dQ = scale dS K
//
// Three pieces of work in two launches, no atomics, no float32 staging of any gradient:
//   1. bwd_self: the self-key terms of target rows' keys (rule 3: a target key is seen by its own row
//      only, so its dk/dv come from that row alone and are written here, final, in bf16).  Its blocks
//      are the last blocks of the dQ grid.
//   2. bwd_dq:   row-stationary, the forward kernel's decomposition: a wave keeps query rows (Q, dO, dQ) in
//      registers and streams the history K/V tiles through LDS.  S^T = K Q^T and dP^T = V dO^T have
//      the query row on the lane, so lse and delta are one register each and dS^T in accumulator layout
//      is directly the k-operand of dQ^T = K^T dS^T.  The self key of a target row is one extra term
//      in the epilogue.  dq is written once.  delta_i = <dO_i, O_i> is formed here, from the dO fragments
//      the wave holds anyway, and left (negated, with -lse/scale) in the workspace for the third kernel.
//   3. bwd_dkdv: key-stationary: a wave owns 32 history keys (K, V fragments and the dK, dV accumulators
//      stay in registers for the whole kernel), the workgroup streams (head, 32-row block) tiles of Q
//      and dO through LDS, shared by its waves.  S = Q K^T and dP = dO V^T have the key on the lane, so
//      P and dS in accumulator layout are directly the k-operand of dV = P^T dO and dK = dS^T Q.
//      dk/dv of history keys are written once.
// S and dP are thus computed twice (7 matrix products instead of 5); in exchange neither dQ nor
// dK/dV ever crosses a workgroup, which removes a float32 accumulator three times the size of q, its
// zero-fill and conversion passes, and an atomic traffic of several GB per call.
// Only history keys are ever visited: target x target and history-row x target-key tiles do not exist
// under the hybrid mask.  Every transposed operand (K^T, Q^T, dO^T) is produced by the LDS transpose
// read from a row-major tile; nothing is transposed when staged.
#include "../../include/mtfm_hta.h"
#include "../../include/mtfm_hta_timing.h"
#include "hta_common.h"
#include "hta_mfma.h"
#include "hta_tiles.h"

namespace hta {
namespace {

__device__ inline float group_sum(float x, int width) {  // sum over aligned groups of `width` lanes
    for (int o = width >> 1; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// ---------------------------------------------------------------------------------------- self keys
// One group of D/8 lanes per (target token, kv head); the group walks the r query heads of the kv head.  A block of
// THREADS threads takes the items block_x * IPB .. of user b.  HBM-bound and small (the target rows only); it has no
// launch of its own: its blocks are the last blocks of the dQ grid, where they fill compute units that the tail of
// that pass leaves idle.
// PW: pointwise weights, p = norm silu(x), ds = norm dp silu'(x) scale (no lse, no delta, `out` is not read).
template <int D, bool PW, int THREADS>
__device__ inline void bwd_self_block(const Params& p, int block_x, int b) {
    constexpr int LPR = D / 8;           // lanes per item, 8 elements (16 bytes) each
    constexpr int IPB = THREADS / LPR;   // items per block
    const int L = p.hist_len[b] + (p.rt_len ? p.rt_len[b] : 0), T = p.n_targets[b];  // L: tokens before the targets
    const int r = p.Hq / p.Hkv;
    const int item = block_x * IPB + threadIdx.x / LPR;  // (target, g) flattened, g fastest
    const int sub = threadIdx.x % LPR;
    const int t = item / p.Hkv, g = item % p.Hkv;
    if (t >= T) return;  // whole lane groups leave together; group_sum only talks inside a group
    const int64_t q_row = (int64_t)p.q_off[b] + (p.layer == 0 ? L + t : t);
    const __bf16* qg = (const __bf16*)p.q;
    const __bf16* dog = (const __bf16*)p.dout;
    const __bf16* og = (const __bf16*)p.out;
    const int64_t kv_off = (((int64_t)p.kv_off[b] + L + t) * p.Hkv + g) * D + sub * 8;
    const bf16x8 kk = *(const bf16x8*)((const __bf16*)p.k + kv_off);
    const bf16x8 vv = *(const bf16x8*)((const __bf16*)p.v + kv_off);
    float kself[8], vself[8], dk_t[8], dv_t[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        kself[j] = (float)kk[j];
        vself[j] = (float)vv[j];
        dk_t[j] = 0.f;
        dv_t[j] = 0.f;
    }
    for (int hh = 0; hh < r; hh++) {
        const int h = g * r + hh;
        const int64_t off = (q_row * p.Hq + h) * D + sub * 8;
        const bf16x8 dov = *(const bf16x8*)(dog + off);
        const bf16x8 ov = PW ? dov : *(const bf16x8*)(og + off);
        const bf16x8 qv = *(const bf16x8*)(qg + off);
        float dof[8], qf[8], part = 0.f, sp = 0.f, dpp = 0.f;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            dof[j] = (float)dov[j];
            qf[j] = (float)qv[j];
            part = fmaf(dof[j], (float)ov[j], part);
            sp = fmaf(qf[j], kself[j], sp);
            dpp = fmaf(dof[j], vself[j], dpp);
        }
        const float sc = group_sum(sp, LPR) * p.scale;
        const float dp = group_sum(dpp, LPR);
        float pw, ds;
        if constexpr (PW) {
            const float sg = 1.f / (1.f + __expf(-sc));
            pw = p.norm * pw_silu(sc, sg);
            ds = p.norm * dp * pw_silu_prime(sc, sg) * p.scale;
        } else {
            const float delta = group_sum(part, LPR);
            const float lse = p.lse[(int64_t)h * p.total_q + q_row];
            pw = __expf(sc - lse);
            ds = pw * (dp - delta) * p.scale;
        }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            dk_t[j] = fmaf(ds, qf[j], dk_t[j]);
            dv_t[j] = fmaf(pw, dof[j], dv_t[j]);
        }
    }
    bf16x8 dk8, dv8;
#pragma unroll
    for (int j = 0; j < 8; j++) {
        dk8[j] = (__bf16)dk_t[j];
        dv8[j] = (__bf16)dv_t[j];
    }
    *(bf16x8*)((__bf16*)p.dk + kv_off) = dk8;
    *(bf16x8*)((__bf16*)p.dv + kv_off) = dv8;
}

// ---------------------------------------------------------------------------------------- dQ
constexpr int BN = 64;  // keys per LDS tile of the dQ kernel

// RT: users with real-time tokens (mask rule 2), handled as in the forward kernel: their keys run through the same
// tile loop, masked per query row with the row's limit; a real-time row gets its own key in the epilogue.
// PW: the pointwise reading of phi2 -- dS = dP o silu'(scale S), scaled by norm * scale at the store; no lse, no
// delta, `out` is not read.  The row statistics the dK/dV pass starts its accumulators from are left as zeros.
// Blocks n_dq .. of the grid are the self-key blocks (bwd_self_block), self_bpu per user.
template <int D, int RB, int NW, bool RT, bool PW = false>
__global__ __launch_bounds__(NW * 64, 2) void bwd_dq_kernel(Params p, int hpb, int n_hc, int tpg, unsigned n_dq, unsigned self_bpu) {
    if (blockIdx.x >= n_dq) {  // uniform for the block, and before any barrier
        const unsigned sb = blockIdx.x - n_dq;
        bwd_self_block<D, PW, NW * 64>(p, (int)(sb % self_bpu), (int)(sb / self_bpu));
        return;
    }
    using ST = KvStage<D, NW>;
    constexpr int NKS = D / 16, NDB = D / 32, NKB = BN / 32;
    static_assert(ST::BN == BN, "tile height");
    // NSTAGE stages of [K tile][V tile], filled by asynchronous global -> LDS copies NSTAGE-1 tiles ahead of their use
    // (two ahead, except for d = 128 where a third stage would cost the second workgroup of the CU).  The compiler
    // never sees a store into this array (the copies are issued from inline assembly), so it neither orders LDS reads
    // against them nor drains them; the counted waits and barriers below do that.
    constexpr int NSTAGE = D <= 64 ? 3 : 2, AHEAD = NSTAGE - 1;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[NSTAGE * ST::BYTES];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    // behind the -lse/scale array: what the S accumulators of rows that do not exist start from in the dK/dV pass
    if (blockIdx.x == 0 && tid == 0) p.neg_lse_s[(int64_t)p.Hq * p.total_q] = -1e30f;
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
    const int tok_shift = p.layer == 0 ? 0 : LK;
    const int64_t q_base = p.q_off[b], kv_base = p.kv_off[b];
    const __bf16* kg = (const __bf16*)p.k;
    const __bf16* vg = (const __bf16*)p.v;
    const float c2 = p.scale * LOG2E;
    const float neg_c2 = -c2;

    const int n_kt = (LK + BN - 1) / BN;
    int nat[NKS], tlo[NDB], thi[NDB];  // per-lane element offsets of the operand fragments inside a swizzled tile
    natural_offsets<D>(nat, lane);
    transposed_offsets<D>(tlo, thi, lane);
    uint32_t voff[ST::COPIES];
    ST::lane_offsets(voff, p.Hkv, wave, lane);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t smem_addr = lds_address(smem);

    // the first K/V tiles are requested before the row operands are loaded and delta is formed: their latencies overlap
    if (n_kt > 0) ST::issue(kg, vg, kv_base, p.Hkv, g, LK, 0, smem_addr, voff, wave_u, lane);
    if (AHEAD > 1 && n_kt > 1) ST::issue(kg, vg, kv_base, p.Hkv, g, LK, 1, smem_addr + ST::BYTES, voff, wave_u, lane);

    // per lane: one query row per row block (clamped past the end; never stored then)
    bf16x8 qf[RB][NKS], dof[RB][NKS];
    float lse2[RB], dl[RB];
    int lim[RB];  // RT: leading keys the lane's row sees
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
        int row = wrow0 + rb * 32 + l32;
        const bool row_live = row < n_rows;
        row = row_live ? row : n_rows - 1;
        const int64_t off = ((q_base + row) * p.Hq + h) * D + 8 * hf;
        float part = 0.f;  // this lane's half of delta = <dO, O>
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            qf[rb][ks] = *(const bf16x8*)((const __bf16*)p.q + off + ks * 16);
            dof[rb][ks] = *(const bf16x8*)((const __bf16*)p.dout + off + ks * 16);
            if constexpr (!PW) part = dot_bf16x8(part, dof[rb][ks], *(const bf16x8*)((const __bf16*)p.out + off + ks * 16));
        }
        const int64_t stat = (int64_t)h * p.total_q + q_base + row;
        const float lse = PW ? 0.f : p.lse[stat];
        const float delta = part + other_half(part);
        lse2[rb] = lse * LOG2E;
        dl[rb] = -delta;
        lim[rb] = RT ? p.lim[q_base + row] : L;
        // every (row, head) belongs to exactly one wave of this kernel: it leaves the row statistics for the dK/dV pass
        if (row_live && hf == 0) {
            p.neg_delta[stat] = -delta;
            p.neg_lse_s[stat] = -lse / p.scale;
        }
    }
    floatx16 dQ[RB][NDB];  // dQ^T: [d (registers)][row (lanes)]
#pragma unroll
    for (int rb = 0; rb < RB; rb++)
#pragma unroll
        for (int db = 0; db < NDB; db++)
#pragma unroll
            for (int v = 0; v < 16; v++) dQ[rb][db][v] = 0.f;

    auto subtile = [&](const __bf16* Ks, const __bf16* Vs, int n_live, int k0) __attribute__((always_inline)) {  // Ks, Vs: first row of the sub-tile (key k0)
        const bool masked = RT && k0 + 32 > L;  // uniform: the sub-tile holds real-time keys (or runs past the end)
        if (masked) {
            bool any = false;
#pragma unroll
            for (int rb = 0; rb < RB; rb++) any = any || lim[rb] > k0;
            if (__builtin_amdgcn_ballot_w64(any) == 0) return;  // no row of this wave sees any key of the sub-tile
        }
        floatx16 S[RB], dP[RB];  // S^T, dP^T: [key (registers)][row (lanes)]
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            const bf16x8 kf = *(const bf16x8*)(Ks + nat[ks]);
            const bf16x8 vf = *(const bf16x8*)(Vs + nat[ks]);
#pragma unroll
            for (int rb = 0; rb < RB; rb++) {
                if (ks == 0) {
                    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    S[rb] = mfma32(kf, qf[rb][ks], zero);
                    dP[rb] = mfma32(vf, dof[rb][ks], zero);
                } else {
                    S[rb] = mfma32(kf, qf[rb][ks], S[rb]);
                    dP[rb] = mfma32(vf, dof[rb][ks], dP[rb]);
                }
            }
        }
        // Register v of the lane holds key 8 (v / 4) + 4 hf + v % 4 of the sub-tile; it is masked when that is >= the
        // number of visible keys, written as 4 hf - visible >= -(8 (v / 4) + v % 4): one subtraction per lane and
        // comparisons with constants, instead of sixteen lane constants kept in registers.
        if (masked) {  // per row: keys at or past the row's limit are not visible (P = 0)
            static_for<0, RB>([&](auto Rb) {
                constexpr int rb = decltype(Rb)::value;
                const int over = 4 * hf - (lim[rb] - k0);
                static_for<0, 16>([&](auto V) {
                    constexpr int v = decltype(V)::value;
                    S[rb][v] = (over >= -(8 * (v / 4) + (v % 4))) ? (PW ? PW_MASKED : -INFINITY) : S[rb][v];
                });
            });
        } else if (n_live < 32) {  // ragged: keys >= L_b are not visible (P = 0)
            const int over = 4 * hf - n_live;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                if (over >= -(8 * (v / 4) + (v % 4))) {
#pragma unroll
                    for (int rb = 0; rb < RB; rb++) S[rb][v] = PW ? PW_MASKED : -INFINITY;
                }
            }
        }
        bf16x8 dsb[RB][2];
#pragma unroll
        for (int rb = 0; rb < RB; rb++)
#pragma unroll
            for (int v = 0; v < 16; v++) {
                if constexpr (PW) {
                    const float sg = pw_sigmoid(S[rb][v], neg_c2);
                    dsb[rb][v / 8][v % 8] = (__bf16)(dP[rb][v] * pw_silu_prime(S[rb][v] * p.scale, sg));
                } else {
                    const float pw = fast_exp2(fmaf(S[rb][v], c2, -lse2[rb]));
                    dsb[rb][v / 8][v % 8] = (__bf16)(pw * (dP[rb][v] + dl[rb]));
                }
            }
        // dQ^T[d][row] += sum_key K[key][d] dS^T[key][row]
#pragma unroll
        for (int db = 0; db < NDB; db++)
#pragma unroll
            for (int s2 = 0; s2 < 2; s2++) {
                const bf16x8 ktf = lds_read_tr_pair(Ks + 16 * s2 * D + tlo[db], Ks + 16 * s2 * D + thi[db]);
#pragma unroll
                for (int rb = 0; rb < RB; rb++) dQ[rb][db] = mfma32(ktf, dsb[rb][s2], dQ[rb][db]);
            }
    };

    // From here on the only vector-memory traffic of the loop are the asynchronous copies, which this code counts
    // itself; the compiler must not be left with pending loads of its own (Q, dO, O, lse) that it would wait for
    // inside the loop.  (The first tiles were requested before those loads.)
    wait_vmem_loads();
    lds_barrier();
    // Tile t is consumed from stage t % NSTAGE while tile t+AHEAD is fetched into stage (t+AHEAD) % NSTAGE, which was
    // last read for tile t-1, i.e. before the barrier that every wave has passed.
    auto tile = [&](int t, auto St) __attribute__((always_inline)) {
        constexpr int st = decltype(St)::value;
        if (t + AHEAD < n_kt)
            ST::issue(kg, vg, kv_base, p.Hkv, g, LK, t + AHEAD, smem_addr + ((st + AHEAD) % NSTAGE) * ST::BYTES, voff, wave_u, lane);
        const __bf16* Ks = (const __bf16*)(smem + st * ST::BYTES);
        const __bf16* Vs = Ks + ST::TILE;
        const int live = LK - t * BN;  // keys of this tile that exist (>= 1)
#pragma unroll
        for (int kb = 0; kb < NKB; kb++) {
            const int n_live = live - kb * 32;
            if (n_live > 0) subtile(Ks + kb * 32 * D, Vs + kb * 32 * D, n_live, t * BN + kb * 32);
        }
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

    // epilogue: self key of target rows (rule 3), scale, store
    __bf16* dqg = (__bf16*)p.dq;
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
        const int row = wrow0 + rb * 32 + l32;
        const bool live = row < n_rows;
        const int tok = tok_shift + row;
        if (live && tok >= L) {
            const int64_t off = ((kv_base + tok) * p.Hkv + g) * D;
            float sp = 0.f, dpp = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ks++) {
                const bf16x8 kk = *(const bf16x8*)(kg + off + ks * 16 + 8 * hf);
                const bf16x8 vv = *(const bf16x8*)(vg + off + ks * 16 + 8 * hf);
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    sp = fmaf((float)qf[rb][ks][j], (float)kk[j], sp);
                    dpp = fmaf((float)dof[rb][ks][j], (float)vv[j], dpp);
                }
            }
            sp += other_half(sp);
            dpp += other_half(dpp);
            float ds;
            if constexpr (PW) {
                ds = dpp * pw_silu_prime(sp * p.scale, pw_sigmoid(sp, neg_c2));
            } else {
                const float pw = fast_exp2(fmaf(sp, c2, -lse2[rb]));
                ds = pw * (dpp + dl[rb]);
            }
#pragma unroll
            for (int db = 0; db < NDB; db++)
#pragma unroll
                for (int v4 = 0; v4 < 4; v4++) {
                    const bf16x4 kk = *(const bf16x4*)(kg + off + db * 32 + 8 * v4 + 4 * hf);
#pragma unroll
                    for (int j = 0; j < 4; j++) dQ[rb][db][4 * v4 + j] = fmaf(ds, (float)kk[j], dQ[rb][db][4 * v4 + j]);
                }
        }
        if (live) {
            __bf16* op = dqg + ((q_base + row) * p.Hq + h) * D;
#pragma unroll
            for (int db = 0; db < NDB; db++)
#pragma unroll
                for (int v4 = 0; v4 < 4; v4++) {
                    bf16x4 o4;
#pragma unroll
                    for (int j = 0; j < 4; j++) o4[j] = (__bf16)(dQ[rb][db][4 * v4 + j] * (PW ? p.scale * p.norm : p.scale));
                    *(bf16x4*)(op + db * 32 + 8 * v4 + 4 * hf) = o4;
                }
        }
    }
}

// ---------------------------------------------------------------------------------------- dK, dV
template <int D, int NW, bool RT>
struct DkdvSmem {
    static constexpr int UPI = 2;      // (head, 32-row block) units per loop iteration, i.e. per workgroup barrier
    static constexpr int NSTAGE = 3;   // iterations resident in LDS: one being consumed, two in flight
    static constexpr int TILE = 32 * D;                 // one unpadded, swizzled 32-row tile (elements)
    // Q, dO, -lse/scale[32], -delta[32]; with real-time tokens also the rows' limits, int[32] (written twice)
    static constexpr size_t UNIT_BYTES = (size_t)2 * TILE * 2 + 2 * 32 * sizeof(float) + (RT ? 256 : 0);
    static constexpr size_t STAGE_BYTES = UPI * UNIT_BYTES;
    static constexpr size_t BYTES = NSTAGE * STAGE_BYTES;
};

// One workgroup per (user, kv head, tile of NW*32 history keys).  Q and dO tiles travel global -> LDS directly
// (no register stop-over), two iterations ahead of their use.
// RT: users with real-time tokens (mask rule 2).  Their keys follow the history keys and are owned by waves like any
// other key; a wave whose 32 keys reach past the history takes the masked instruction stream, where a weight
// survives only if the key lies below the row's limit (p.lim, staged with the row statistics) or is the row's own
// token (the own key of a real-time row; target rows' own keys are the business of bwd_self_block).
// PW: the pointwise reading of phi2 -- P = silu(scale S), dS = dP o silu'(scale S); the staged row statistics are
// zeros for rows that exist (the sentinel for rows that do not still removes them), norm is applied at the store.
template <int D, int NW, bool RT, bool PW = false>
__global__ __launch_bounds__(NW * 64, D > 64 ? 1 : 2) void bwd_dkdv_kernel(Params p, int tpg, unsigned per_xcd) {
    using SM = DkdvSmem<D, NW, RT>;
    static_assert(!RT || NW >= 2 * SM::UPI, "waves UPI .. 2 UPI - 1 copy the rows' limits");
    constexpr int UPI = SM::UPI, NSTAGE = SM::NSTAGE;
    constexpr int NKS = D / 16, NDB = D / 32;
    constexpr int CPR = D / 8;                  // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;               // rows covered by one wave-wide 1 KB copy
    constexpr int IPT = 32 / RPI;               // copies per tile
    constexpr int IPW = (IPT + NW - 1) / NW;    // copies per tile issued by one wave (the last may be idle)
    constexpr int COPIES = UPI * 2 * IPW;       // direct copies per wave and iteration (when the wave takes part)
    static_assert(IPT % NW == 0 || IPT < NW, "tile copies must split evenly over the waves");
    static_assert(UPI <= NW, "wave uu copies the row statistics of unit uu");
    // One array per stage: copies in flight into one stage and reads from another are then provably disjoint, so the
    // compiler need not drain the copies before every LDS read.
    __shared__ __attribute__((aligned(1024))) unsigned char stage0[SM::STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char stage1[SM::STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char stage2[SM::STAGE_BYTES];
    static_assert(NSTAGE == 3, "three stage arrays");
    auto stage_ptr = [&](auto St) -> unsigned char* {
        constexpr int st = decltype(St)::value % 3;
        if constexpr (st == 0) return stage0;
        if constexpr (st == 1) return stage1;
        return stage2;
    };

    __shared__ int s_item;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;

    // one work item: a (user, kv head, key tile) triple
    auto process = [&](unsigned id) {
    const WorkItem w = decode_work(id, p.batch * p.Hkv, p.Hkv, tpg);
    if (!w.valid) return;
    const int b = scheduled_user(p, w.user_slot), g = w.y;
    const int L = p.hist_len[b], T = p.n_targets[b];
    const int LK = L + (RT ? p.rt_len[b] : 0);  // keys that receive gradient here: history, then real-time
    const int key0 = w.tile * (NW * 32);
    if (key0 >= LK) return;  // uniform: this key tile does not exist for the user
    const int n_rows = p.layer == 0 ? LK + T : T;
    const int tok_shift = p.layer == 0 ? 0 : LK;  // token index of query row 0
    const int r = p.Hq / p.Hkv;
    const int64_t q_base = p.q_off[b], kv_base = p.kv_off[b];
    const float c2 = p.scale * LOG2E;
    const int kw = key0 + wave * 32;        // first key of this wave
    const bool wave_live = kw < LK;         // a wave past the last key only helps staging
    const bool key_live = kw + l32 < LK;
    const bool wave_ragged = kw + 32 > L;   // past the end, or (RT) into the real-time keys: masked instruction stream
    const bool copies = IPT >= NW || wave < IPT;   // does this wave issue tile copies?

    // per-lane element offsets into a swizzled tile
    int nat_off[NKS];   // row l32, chunk 2*ks + hf: fragments with the row on the lane
#pragma unroll
    for (int ks = 0; ks < NKS; ks++) nat_off[ks] = l32 * D + (((2 * ks + hf) ^ swizzle<D>(l32)) << 3);
    // transposed fragments: rows 4*hf + (lane%16)/4 and 8 below (+16 per k-step, which leaves the swizzle
    // unchanged), 4 elements at column 32*db + 16*((lane/16)%2) + 4*(lane%4)
    int tr_lo[NDB], tr_hi[NDB];
    {
        const int pl = lane & 15, trow = 4 * hf + (pl >> 2);
#pragma unroll
        for (int db = 0; db < NDB; db++) {
            const int chunk = 4 * db + 2 * ((lane >> 4) & 1) + ((pl & 3) >> 1);
            tr_lo[db] = trow * D + ((chunk ^ swizzle<D>(trow)) << 3) + 4 * (pl & 1);
            tr_hi[db] = (trow + 8) * D + ((chunk ^ swizzle<D>(trow + 8)) << 3) + 4 * (pl & 1);
        }
    }

    // stationary operands: K and V rows of the wave's keys (B operand of S = Q K^T and dP = dO V^T)
    bf16x8 kf[NKS], vf[NKS];
    {
        const int key = key_live ? kw + l32 : LK - 1;
        const int64_t off = ((kv_base + key) * p.Hkv + g) * D + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            kf[ks] = *(const bf16x8*)((const __bf16*)p.k + off + ks * 16);
            vf[ks] = *(const bf16x8*)((const __bf16*)p.v + off + ks * 16);
        }
    }
    floatx16 dK[NDB], dV[NDB];  // [key (registers)][d (lanes)]
#pragma unroll
    for (int db = 0; db < NDB; db++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
            dK[db][v] = 0.f;
            dV[db][v] = 0.f;
        }

    const int n_rb = (n_rows + 31) / 32;
    const int n_units = n_rb * r;  // unit u = (32-row block u / r, head g*r + u % r)
    const int n_iter = (n_units + UPI - 1) / UPI;  // 0 for a user without query rows: dK = dV = 0 is still written

    // Q and dO tiles of iteration `it` -> stage it % NSTAGE.  Copy j of a tile covers rows j*RPI .. j*RPI+RPI-1:
    // lane i lands at chunk position i % CPR of row j*RPI + i / CPR, so it fetches the chunk that belongs there.
    // The calls come in the order it = 0, 1, 2, ...; the unit the next call starts with is kept in (iss_rb, iss_hh).
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint32_t tile_voff[IPW];  // byte offset of the lane's chunk from the first element of (row0, head h)
#pragma unroll
    for (int jj = 0; jj < IPW; jj++) {
        const int trow = (wave + jj * NW) * RPI + lane / CPR;
        tile_voff[jj] = (uint32_t)((trow * p.Hq * D + (((lane % CPR) ^ swizzle<D>(trow)) << 3)) * 2);
    }
    const float* stat_lane = (hf == 0 ? p.neg_lse_s : p.neg_delta) + q_base + l32;
    const int32_t* lim_lane = RT ? p.lim + q_base + l32 : nullptr;  // both halves of the wave fetch the same 32 limits
    int iss_rb = 0, iss_hh = 0;
    auto issue_tiles = [&](auto St) {
        const uint32_t stage = lds_address(stage_ptr(St));
#pragma unroll
        for (int uu = 0; uu < UPI; uu++) {
            // a unit past the last one repeats the last one, with no weight
            const bool past = iss_rb >= n_rb;
            const int rb = past ? n_rb - 1 : iss_rb, hh = past ? r - 1 : iss_hh;
            const int row0 = rb * 32, h = g * r + hh;
            const bool whole = !past && row0 + 32 <= n_rows;  // every row exists: no per-lane address arithmetic
            const uint32_t unit = stage + uu * (uint32_t)SM::UNIT_BYTES;
            const int64_t ubase = ((q_base + row0) * p.Hq + h) * (int64_t)D;
            if (whole) {
#pragma unroll
                for (int jj = 0; jj < (copies ? IPW : 0); jj++) {
                    const uint32_t dst = unit + (uint32_t)(wave_u + jj * NW) * 1024u;
                    copy16_global_to_lds_at((const __bf16*)p.q + ubase, tile_voff[jj], dst);
                    copy16_global_to_lds_at((const __bf16*)p.dout + ubase, tile_voff[jj], dst + (uint32_t)SM::TILE * 2u);
                }
                if (wave_u == uu) copy4_global_to_lds_at(stat_lane + ((int64_t)h * p.total_q + row0), unit + 4u * (uint32_t)SM::TILE);
                if (RT && wave_u == uu + UPI) copy4_global_to_lds_at(lim_lane + row0, unit + 4u * (uint32_t)SM::TILE + 256u);
            } else {
#pragma unroll
                for (int jj = 0; jj < (copies ? IPW : 0); jj++) {
                    const int trow = (wave + jj * NW) * RPI + lane / CPR;
                    int row = row0 + trow;
                    row = row < n_rows ? row : n_rows - 1;  // rows past the end repeat the last row, with no weight
                    const int chunk = (lane % CPR) ^ swizzle<D>(trow);
                    const int64_t off = ((q_base + row) * p.Hq + h) * D + chunk * 8;
                    const uint32_t dst = unit + (uint32_t)(wave_u + jj * NW) * 1024u;
                    copy16_global_to_lds_at((const __bf16*)p.q + off, dst);
                    copy16_global_to_lds_at((const __bf16*)p.dout + off, dst + (uint32_t)SM::TILE * 2u);
                }
                // A row that does not exist starts from the sentinel behind the -lse/scale array, a huge negative
                // number: its weights P = exp(scale * that) are exactly 0, and so is all it would add to dK and dV.
                if (wave_u == uu) {
                    int row = row0 + l32;
                    const bool dead = past || row >= n_rows;
                    row = row < n_rows ? row : n_rows - 1;
                    const int64_t idx = (int64_t)h * p.total_q + q_base + row;
                    const float* src = hf == 0 ? p.neg_lse_s + (dead ? (int64_t)p.Hq * p.total_q : idx) : p.neg_delta + idx;
                    copy4_global_to_lds_at(src, unit + 4u * (uint32_t)SM::TILE);
                }
                if (RT && wave_u == uu + UPI) {
                    int row = row0 + l32;
                    row = row < n_rows ? row : n_rows - 1;
                    copy4_global_to_lds_at(p.lim + q_base + row, unit + 4u * (uint32_t)SM::TILE + 256u);
                }
            }
            if (!past && ++iss_hh == r) {
                iss_hh = 0;
                iss_rb++;
            }
        }
    };
    // wait until at most the copies this wave has issued for its K most recent iterations are outstanding
    auto wait_all_but_iterations = [&](auto Kc) {
        constexpr int K = decltype(Kc)::value;
        const bool extra = wave < UPI || (RT && wave < 2 * UPI);  // one more copy per iteration: statistics, or limits
        if (copies) {
            if (extra) wait_vmem_outstanding<K * (COPIES + 1)>(); else wait_vmem_outstanding<K * COPIES>();
        } else {
            if (extra) wait_vmem_outstanding<K>(); else wait_vmem_outstanding<0>();
        }
    };
    const std::integral_constant<int, 0> c0{};
    const std::integral_constant<int, 1> c1{};

    // The wave's work on one (head, 32-row block) unit against its 32 keys, in four steps that the loop below
    // interleaves across units: fetch the operands, S and dP, the weights, the two accumulations.
    struct Operands {
        bf16x8 qa[NKS], da[NKS];
        floatx16 S, dP;  // [row (registers)][key (lanes)]
    };
    struct Transposed {
        bf16x8 dot[NDB][2], qt[NDB][2];
    };
    auto load_operands = [&](const unsigned char* ubase, Operands& o) {
        const __bf16* Qs = (const __bf16*)ubase;
        const __bf16* dOs = Qs + SM::TILE;
        const float* ss = (const float*)(dOs + SM::TILE);
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            o.qa[ks] = *(const bf16x8*)(Qs + nat_off[ks]);
            o.da[ks] = *(const bf16x8*)(dOs + nat_off[ks]);
        }
        // accumulators start from -lse/scale and -delta of their rows (registers 4j..4j+3 hold rows 8j+4hf .. +3)
        floatx4 l4[4], d4[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            l4[j] = *(const floatx4*)(ss + 8 * j + 4 * hf);
            d4[j] = *(const floatx4*)(ss + 32 + 8 * j + 4 * hf);
        }
        o.S = __builtin_shufflevector(__builtin_shufflevector(l4[0], l4[1], 0, 1, 2, 3, 4, 5, 6, 7),
                                      __builtin_shufflevector(l4[2], l4[3], 0, 1, 2, 3, 4, 5, 6, 7), 0, 1, 2, 3, 4, 5, 6, 7, 8,
                                      9, 10, 11, 12, 13, 14, 15);
        o.dP = __builtin_shufflevector(__builtin_shufflevector(d4[0], d4[1], 0, 1, 2, 3, 4, 5, 6, 7),
                                       __builtin_shufflevector(d4[2], d4[3], 0, 1, 2, 3, 4, 5, 6, 7), 0, 1, 2, 3, 4, 5, 6, 7,
                                       8, 9, 10, 11, 12, 13, 14, 15);
    };
    auto scores = [&](Operands& o) {
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            o.S = mfma32(o.qa[ks], kf[ks], o.S);     // S - lse/scale
            o.dP = mfma32(o.da[ks], vf[ks], o.dP);   // dP - delta
        }
    };
    auto load_transposed = [&](const unsigned char* ubase, Transposed& f) {
        const __bf16* Qs = (const __bf16*)ubase;
        const __bf16* dOs = Qs + SM::TILE;
#pragma unroll
        for (int db = 0; db < NDB; db++)
#pragma unroll
            for (int s2 = 0; s2 < 2; s2++) {
                f.dot[db][s2] = lds_read_tr_pair(dOs + tr_lo[db] + 16 * s2 * D, dOs + tr_hi[db] + 16 * s2 * D);
                f.qt[db][s2] = lds_read_tr_pair(Qs + tr_lo[db] + 16 * s2 * D, Qs + tr_hi[db] + 16 * s2 * D);
            }
    };
    struct Weights {
        bf16x8 pb[2], dsb[2];
    };
    // `ubase`, `u`: the unit's place in LDS and its number (used by the masked stream only)
    auto weights = [&](const Operands& o, Weights& wt, auto ragged, const unsigned char* ubase, int u) {
        constexpr bool MASKED = decltype(ragged)::value;
        int limv[16];     // RT: limits of the unit's rows, register v <-> row 8(v/4) + 4 hf + v%4
        int self_row = 0; // RT: the row of the unit whose own token is this lane's key (if it is one of its 32 rows)
        if constexpr (MASKED && RT) {
            typedef int int4v __attribute__((ext_vector_type(4)));
            const int* ls = (const int*)(ubase + (size_t)4 * SM::TILE + 256);
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int4v l4 = *(const int4v*)(ls + 8 * j + 4 * hf);
#pragma unroll
                for (int i = 0; i < 4; i++) limv[4 * j + i] = l4[i];
            }
            self_row = kw + l32 - tok_shift - (u / r) * 32;
        }
        if constexpr (PW) {
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const float sg = pw_sigmoid(o.S[v], -c2);
                const float x = o.S[v] * p.scale;
                float pw = pw_silu(x, sg), sp = pw_silu_prime_of(pw, sg);
                if constexpr (MASKED && RT) {
                    const int key = kw + l32;
                    const bool vis = key < limv[v] || (key_live && self_row == 8 * (v / 4) + 4 * hf + (v % 4));
                    pw = vis ? pw : 0.f;
                    sp = vis ? sp : 0.f;
                } else if constexpr (MASKED) {  // keys past the history carry no weight
                    pw = key_live ? pw : 0.f;
                    sp = key_live ? sp : 0.f;
                }
                wt.pb[v / 8][v % 8] = (__bf16)pw;
                wt.dsb[v / 8][v % 8] = (__bf16)(sp * o.dP[v]);
            }
            return;
        }
#pragma unroll
        for (int v = 0; v < 16; v++) {
            float pw = fast_exp2(o.S[v] * c2);
            if constexpr (MASKED && RT) {
                const int key = kw + l32;
                const bool vis = key < limv[v] || (key_live && self_row == 8 * (v / 4) + 4 * hf + (v % 4));
                pw = vis ? pw : 0.f;
            } else if constexpr (MASKED) {
                pw = key_live ? pw : 0.f;  // keys past the history carry no weight
            }
            wt.pb[v / 8][v % 8] = (__bf16)pw;
            wt.dsb[v / 8][v % 8] = (__bf16)(pw * o.dP[v]);
        }
    };
    // dV[key][d] += P^T[key][row] dO[row][d];  dK[key][d] += dS^T[key][row] Q[row][d]
    auto accumulate = [&](const Weights& wt, const Transposed& f) {
#pragma unroll
        for (int db = 0; db < NDB; db++)
#pragma unroll
            for (int s2 = 0; s2 < 2; s2++) {
                dV[db] = mfma32(wt.pb[s2], f.dot[db][s2], dV[db]);
                dK[db] = mfma32(wt.dsb[s2], f.qt[db][s2], dK[db]);
            }
    };

    const std::integral_constant<int, 0> st0{};
    const std::integral_constant<int, 1> st1{};
    const std::integral_constant<int, 2> st2{};
    static_assert(UPI == 2, "the loop below is written out for two units per iteration");
    // prologue: all three stages requested while the K/V fragments are still on their way (one memory latency instead
    // of two at the start of every item).  From the wait on, the only vector-memory traffic of the loop are the
    // asynchronous copies, which this code counts itself; the compiler must not be left with pending loads of its own
    // that it would wait for inside the loop.
    if (n_iter > 0) issue_tiles(st0);
    if (n_iter > 1) issue_tiles(st1);
    if (n_iter > 2) issue_tiles(st2);
    wait_vmem_loads();
    lds_barrier();

    // Iteration `it` consumes stage it % 3.  Its barrier sits in the middle of the second unit, after the last LDS read
    // of the stage: behind it the stage is refilled for iteration it+3 and the operands of iteration it+1 are fetched,
    // both while the second unit's accumulations keep the matrix unit busy.
    auto run = [&](auto ragged) {
        Operands cur;
        load_operands(stage_ptr(st0), cur);
        auto iteration = [&](int it, auto St) {
            constexpr int st = decltype(St)::value;
            const unsigned char* base = stage_ptr(St);
            Operands nxt;
            Transposed f;
            Weights wt;
            if constexpr (RT) {
                scores(cur);
                load_transposed(base, f);
                weights(cur, wt, ragged, base, it * UPI);
                load_operands(base + SM::UNIT_BYTES, nxt);
                accumulate(wt, f);
                scores(nxt);
                load_transposed(base + SM::UNIT_BYTES, f);
                weights(nxt, wt, ragged, base + SM::UNIT_BYTES, it * UPI + 1);
            } else {
                // The second unit's S and dP are requested before the first unit's weights are formed, and the first
                // unit's accumulations come after the second unit's weights: each block of vector work then has matrix
                // instructions of the other unit in the stream around it (3 % at d = 64, 6 % at d = 128; the
                // real-time variant keeps the shorter live ranges, it has no registers to spare).
                Weights wt0;
                scores(cur);
                load_operands(base + SM::UNIT_BYTES, nxt);
                weights(cur, wt0, ragged, base, it * UPI);
                scores(nxt);
                load_transposed(base, f);
                weights(nxt, wt, ragged, base + SM::UNIT_BYTES, it * UPI + 1);
                accumulate(wt0, f);
                load_transposed(base + SM::UNIT_BYTES, f);
            }
            // copies of iteration it+1 must have landed; those of it+2 may stay in flight
            if (it + 2 < n_iter) wait_all_but_iterations(c1); else wait_all_but_iterations(c0);
            lds_barrier();
            if (it + 3 < n_iter) issue_tiles(St);
            // (behind the last iteration this reads a stage that holds nothing new; the values are not used)
            load_operands(stage_ptr(std::integral_constant<int, (st + 1) % 3>{}), cur);
            accumulate(wt, f);
        };
        for (int it = 0; it < n_iter; it += 3) {
            iteration(it, st0);
            if (it + 1 < n_iter) iteration(it + 1, st1);
            if (it + 2 < n_iter) iteration(it + 2, st2);
        }
    };
    // a wave past the history only helps staging: same waits, same barriers, same copies
    auto run_idle = [&]() {
        auto iteration = [&](int it, auto St) {
            if (it + 2 < n_iter) wait_all_but_iterations(c1); else wait_all_but_iterations(c0);
            lds_barrier();
            if (it + 3 < n_iter) issue_tiles(St);
        };
        for (int it = 0; it < n_iter; it += 3) {
            iteration(it, st0);
            if (it + 1 < n_iter) iteration(it + 1, st1);
            if (it + 2 < n_iter) iteration(it + 2, st2);
        }
    };
    if (n_iter > 0) {
        if (!wave_live) run_idle();
        else if (wave_ragged) run(std::true_type{});
        else run(std::false_type{});
    }

    // write the wave's 32 key rows: lanes cover 32 consecutive d
    if (wave_live) {
        __bf16* dkg = (__bf16*)p.dk;
        __bf16* dvg = (__bf16*)p.dv;
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int key = kw + 8 * (v / 4) + 4 * hf + (v % 4);
            if (key < LK) {
                const int64_t off = ((kv_base + key) * p.Hkv + g) * D + l32;
#pragma unroll
                for (int db = 0; db < NDB; db++) {
                    dkg[off + db * 32] = (__bf16)(dK[db][v] * (PW ? p.scale * p.norm : p.scale));
                    dvg[off + db * 32] = (__bf16)(PW ? dV[db][v] * p.norm : dV[db][v]);
                }
            }
        }
    }
    };  // process

    // persistent workgroup: items come from the work counters until all lists are exhausted
    const int xcd = blockIdx.x % N_XCD;
    unsigned taken = 0;
    if (tid == 0) taken = queue_take_ahead(p.queue, xcd);
    for (;;) {
        if (tid == 0) s_item = queue_resolve(p.queue, xcd, taken, per_xcd);
        __syncthreads();
        const int id = s_item;
        if (id < 0) break;
        if (tid == 0) taken = queue_take_ahead(p.queue, xcd);
        process((unsigned)id);
        __syncthreads();  // the stages and s_item are free again
    }
}

// ---------------------------------------------------------------------------------------- dK, dV: few query rows
// The same pass for batches whose users have few query rows (a target-only layer: the candidates of a user against a
// long history).  bwd_dkdv_kernel streams the rows of a user past every 128-key tile again; with a handful of row
// blocks that is a prologue, a drained pipeline and an epilogue around four to eight iterations.  Here a workgroup
// takes a whole (user, kv head): it stages ALL (head, 32-row block) units of Q and dO in LDS once (at most MAX_UNITS of
// them, which is what the host checks), and then its waves walk the keys, 32 per wave and pass, each on its own: K/V
// fragments from global memory, every unit from LDS, dK/dV stored -- no barrier, no copy and no counted wait inside the
// key loop, and waves that drift apart.  Twelve waves, three per SIMD, one unit in flight per wave (168 registers):
// measured against eight waves with two units interleaved per wave, as bwd_dkdv_kernel does it, the third wave hides
// more than the interleaving (dK/dV of a 512 x 2048 x 128 target layer 1.21 against 1.30 ms; streaming kernel 1.33).
// Softmax weights without real-time tokens only (the callers that need the other readings take the streaming kernel).
template <int D, int NW>
struct DkdvResident {
    static constexpr int MAX_UNITS = 16;
    static constexpr int TILE = 32 * D;                                          // elements of a 32-row tile
    static constexpr size_t UNIT_BYTES = (size_t)2 * TILE * 2 + 2 * 32 * sizeof(float);  // Q, dO, -lse/scale[32], -delta[32]
    static constexpr size_t BYTES = MAX_UNITS * UNIT_BYTES;
};

template <int D, int NW>
__global__ __launch_bounds__(NW * 64, 3) void bwd_dkdv_resident_kernel(Params p, unsigned per_xcd) {
    using SM = DkdvResident<D, NW>;
    constexpr int NKS = D / 16, NDB = D / 32;
    constexpr int CPR = D / 8;      // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;   // rows covered by one wave-wide 1 KB copy
    constexpr int IPT = 32 / RPI;   // copies per tile
    __shared__ __attribute__((aligned(1024))) unsigned char units[SM::BYTES];
    __shared__ int s_item;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int r = p.Hq / p.Hkv;
    const float c2 = p.scale * LOG2E;

    // per-lane element offsets into a swizzled tile (as in bwd_dkdv_kernel)
    int nat_off[NKS], tr_lo[NDB], tr_hi[NDB];
    natural_offsets<D>(nat_off, lane);
    transposed_offsets<D>(tr_lo, tr_hi, lane);
    // copy j of a tile covers rows j*RPI .. j*RPI+RPI-1: byte offset of the lane's chunk from (row0, head h)
    uint32_t tile_voff[IPT];
#pragma unroll
    for (int j = 0; j < IPT; j++) {
        const int trow = j * RPI + lane / CPR;
        tile_voff[j] = (uint32_t)((trow * p.Hq * D + (((lane % CPR) ^ swizzle<D>(trow)) << 3)) * 2);
    }

    struct Operands {
        bf16x8 qa[NKS], da[NKS];
        floatx16 S, dP;  // [row (registers)][key (lanes)]
    };
    struct Transposed {
        bf16x8 dot[NDB][2], qt[NDB][2];
    };
    struct Weights {
        bf16x8 pb[2], dsb[2];
    };

    auto process = [&](unsigned id) {
        const WorkItem w = decode_work(id, p.batch * p.Hkv, p.Hkv, 1);
        if (!w.valid) return;
        const int b = scheduled_user(p, w.user_slot), g = w.y;
        const int LK = p.hist_len[b], T = p.n_targets[b];
        if (LK <= 0) return;  // no key receives a gradient here
        const int n_rows = p.layer == 0 ? LK + T : T;
        const int n_rb = (n_rows + 31) / 32;
        // unit u = (32-row block u / r, head g*r + u % r).  (The launch is chosen from the caller's bounds on the rows of a
        // user; should a user exceed them, the clamp keeps the staging inside LDS.)
        const int n_units = min(n_rb * r, SM::MAX_UNITS);
        const int64_t q_base = p.q_off[b], kv_base = p.kv_off[b];

        // ---- stage every unit: wave u % NW brings unit u (2 * IPT tile copies and the row statistics)
        const uint32_t lds0 = lds_address(units);
        for (int u = wave_u; u < n_units; u += NW) {
            const int rb = u / r, h = g * r + u % r, row0 = rb * 32;
            const uint32_t unit = lds0 + (uint32_t)u * (uint32_t)SM::UNIT_BYTES;
            const bool whole = row0 + 32 <= n_rows;  // every row exists: no per-lane address arithmetic
            if (whole) {
                const int64_t ubase = ((q_base + row0) * p.Hq + h) * (int64_t)D;
#pragma unroll
                for (int j = 0; j < IPT; j++) {
                    copy16_global_to_lds_at((const __bf16*)p.q + ubase, tile_voff[j], unit + (uint32_t)j * 1024u);
                    copy16_global_to_lds_at((const __bf16*)p.dout + ubase, tile_voff[j], unit + (uint32_t)SM::TILE * 2u + (uint32_t)j * 1024u);
                }
                const float* stat = (hf == 0 ? p.neg_lse_s : p.neg_delta) + ((int64_t)h * p.total_q + q_base + row0 + l32);
                copy4_global_to_lds_at(stat, unit + 4u * (uint32_t)SM::TILE);
            } else {
#pragma unroll
                for (int j = 0; j < IPT; j++) {
                    const int trow = j * RPI + lane / CPR;
                    int row = row0 + trow;
                    row = row < n_rows ? row : n_rows - 1;  // rows past the end repeat the last row, with no weight
                    const int chunk = (lane % CPR) ^ swizzle<D>(trow);
                    const int64_t off = ((q_base + row) * p.Hq + h) * D + chunk * 8;
                    copy16_global_to_lds_at((const __bf16*)p.q + off, unit + (uint32_t)j * 1024u);
                    copy16_global_to_lds_at((const __bf16*)p.dout + off, unit + (uint32_t)SM::TILE * 2u + (uint32_t)j * 1024u);
                }
                // a row that does not exist starts from the sentinel behind the -lse/scale array: P = 0 exactly
                int row = row0 + l32;
                const bool dead = row >= n_rows;
                row = row < n_rows ? row : n_rows - 1;
                const int64_t idx = (int64_t)h * p.total_q + q_base + row;
                const float* src = hf == 0 ? p.neg_lse_s + (dead ? (int64_t)p.Hq * p.total_q : idx) : p.neg_delta + idx;
                copy4_global_to_lds_at(src, unit + 4u * (uint32_t)SM::TILE);
            }
        }
        wait_vmem_loads();
        lds_barrier();

        auto unit_ptr = [&](int u) { return units + (size_t)u * SM::UNIT_BYTES; };
        // ---- the keys, 32 per wave and pass
        for (int k0 = wave * 32; k0 < LK; k0 += NW * 32) {
            const int kw = k0;
            const bool key_live = kw + l32 < LK;
            const bool ragged = kw + 32 > LK;
            bf16x8 kf[NKS], vf[NKS];
            {
                const int key = key_live ? kw + l32 : LK - 1;
                const int64_t off = ((kv_base + key) * p.Hkv + g) * D + 8 * hf;
#pragma unroll
                for (int ks = 0; ks < NKS; ks++) {
                    kf[ks] = *(const bf16x8*)((const __bf16*)p.k + off + ks * 16);
                    vf[ks] = *(const bf16x8*)((const __bf16*)p.v + off + ks * 16);
                }
            }
            floatx16 dK[NDB], dV[NDB];  // [key (registers)][d (lanes)]
#pragma unroll
            for (int db = 0; db < NDB; db++)
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    dK[db][v] = 0.f;
                    dV[db][v] = 0.f;
                }
            auto load_operands = [&](const unsigned char* ubase, Operands& o) {
                const __bf16* Qs = (const __bf16*)ubase;
                const __bf16* dOs = Qs + SM::TILE;
                const float* ss = (const float*)(dOs + SM::TILE);
#pragma unroll
                for (int ks = 0; ks < NKS; ks++) {
                    o.qa[ks] = *(const bf16x8*)(Qs + nat_off[ks]);
                    o.da[ks] = *(const bf16x8*)(dOs + nat_off[ks]);
                }
                // accumulators start from -lse/scale and -delta of their rows (registers 4j..4j+3 hold rows 8j+4hf .. +3)
                floatx4 l4[4], d4[4];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    l4[j] = *(const floatx4*)(ss + 8 * j + 4 * hf);
                    d4[j] = *(const floatx4*)(ss + 32 + 8 * j + 4 * hf);
                }
                o.S = __builtin_shufflevector(__builtin_shufflevector(l4[0], l4[1], 0, 1, 2, 3, 4, 5, 6, 7),
                                              __builtin_shufflevector(l4[2], l4[3], 0, 1, 2, 3, 4, 5, 6, 7), 0, 1, 2, 3, 4, 5, 6,
                                              7, 8, 9, 10, 11, 12, 13, 14, 15);
                o.dP = __builtin_shufflevector(__builtin_shufflevector(d4[0], d4[1], 0, 1, 2, 3, 4, 5, 6, 7),
                                               __builtin_shufflevector(d4[2], d4[3], 0, 1, 2, 3, 4, 5, 6, 7), 0, 1, 2, 3, 4, 5, 6,
                                               7, 8, 9, 10, 11, 12, 13, 14, 15);
            };
            auto scores = [&](Operands& o) {
#pragma unroll
                for (int ks = 0; ks < NKS; ks++) {
                    o.S = mfma32(o.qa[ks], kf[ks], o.S);     // S - lse/scale
                    o.dP = mfma32(o.da[ks], vf[ks], o.dP);   // dP - delta
                }
            };
            auto load_transposed = [&](const unsigned char* ubase, Transposed& f) {
                const __bf16* Qs = (const __bf16*)ubase;
                const __bf16* dOs = Qs + SM::TILE;
#pragma unroll
                for (int db = 0; db < NDB; db++)
#pragma unroll
                    for (int s2 = 0; s2 < 2; s2++) {
                        f.dot[db][s2] = lds_read_tr_pair(dOs + tr_lo[db] + 16 * s2 * D, dOs + tr_hi[db] + 16 * s2 * D);
                        f.qt[db][s2] = lds_read_tr_pair(Qs + tr_lo[db] + 16 * s2 * D, Qs + tr_hi[db] + 16 * s2 * D);
                    }
            };
            auto weights = [&](const Operands& o, Weights& wt) {
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    float pw = fast_exp2(o.S[v] * c2);
                    if (ragged) pw = key_live ? pw : 0.f;  // keys past the history carry no weight
                    wt.pb[v / 8][v % 8] = (__bf16)pw;
                    wt.dsb[v / 8][v % 8] = (__bf16)(pw * o.dP[v]);
                }
            };
            // dV[key][d] += P^T[key][row] dO[row][d];  dK[key][d] += dS^T[key][row] Q[row][d]
            auto accumulate = [&](const Weights& wt, const Transposed& f) {
#pragma unroll
                for (int db = 0; db < NDB; db++)
#pragma unroll
                    for (int s2 = 0; s2 < 2; s2++) {
                        dV[db] = mfma32(wt.pb[s2], f.dot[db][s2], dV[db]);
                        dK[db] = mfma32(wt.dsb[s2], f.qt[db][s2], dK[db]);
                    }
            };
            // one unit after the other: the other two waves of the SIMD fill what this one waits for
            {
                Operands cur;
                Transposed f;
                Weights wt;
                for (int u = 0; u < n_units; u++) {
                    load_operands(unit_ptr(u), cur);
                    scores(cur);
                    load_transposed(unit_ptr(u), f);
                    weights(cur, wt);
                    accumulate(wt, f);
                }
            }
            // write the wave's 32 key rows: lanes cover 32 consecutive d
            __bf16* dkg = (__bf16*)p.dk;
            __bf16* dvg = (__bf16*)p.dv;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int key = kw + 8 * (v / 4) + 4 * hf + (v % 4);
                if (key < LK) {
                    const int64_t off = ((kv_base + key) * p.Hkv + g) * D + l32;
#pragma unroll
                    for (int db = 0; db < NDB; db++) {
                        dkg[off + db * 32] = (__bf16)(dK[db][v] * p.scale);
                        dvg[off + db * 32] = (__bf16)dV[db][v];
                    }
                }
            }
        }
    };  // process

    // persistent workgroup, as in bwd_dkdv_kernel
    const int xcd = blockIdx.x % N_XCD;
    unsigned taken = 0;
    if (tid == 0) taken = queue_take_ahead(p.queue, xcd);
    for (;;) {
        if (tid == 0) s_item = queue_resolve(p.queue, xcd, taken, per_xcd);
        __syncthreads();
        const int id = s_item;
        if (id < 0) break;
        if (tid == 0) taken = queue_take_ahead(p.queue, xcd);
        process((unsigned)id);
        __syncthreads();  // the staged units and s_item are free again
    }
}

int gcd_i(int a, int b) { return b == 0 ? a : gcd_i(b, a % b); }

template <int D, int RB, int NW>
hipError_t launch_dq(const Params& p, hipStream_t s) {
    const int r = p.Hq / p.Hkv;
    const int hpb = gcd_i(r, NW);
    const int n_hc = r / hpb;
    const int BM = (NW / hpb) * RB * 32;
    const int64_t rows = max_query_rows(p);
    if (rows <= 0) return hipSuccess;
    const int64_t n_rt = (rows + BM - 1) / BM;
    const int64_t n_blocks = work_grid((int64_t)p.batch * p.Hkv * n_hc, n_rt);
    // the self-key blocks: (target, kv head) items of every user, NW * 64 / (D / 8) per block
    constexpr int IPB = NW * 64 / (D / 8);
    const int64_t self_bpu = ((int64_t)p.max_targets * p.Hkv + IPB - 1) / IPB;
    const int64_t n_self = self_bpu * p.batch;
    if (n_blocks + n_self >= (1ll << 31)) return hipErrorInvalidValue;
    auto kernel = p.pointwise ? (p.rt_len ? bwd_dq_kernel<D, RB, NW, true, true> : bwd_dq_kernel<D, RB, NW, false, true>)
                  : p.rt_len  ? bwd_dq_kernel<D, RB, NW, true> : bwd_dq_kernel<D, RB, NW, false>;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(n_blocks + n_self)), dim3(NW * 64), 0, s, p, hpb, n_hc, (int)n_rt,
                       (unsigned)n_blocks, (unsigned)(self_bpu > 0 ? self_bpu : 1));
    return hipGetLastError();
}

template <int D, int NW, bool RT, bool PW = false>
hipError_t launch_dkdv_as(const Params& p, hipStream_t s) {
    const int64_t keys = max_lead_keys(p);
    if (keys <= 0) return hipSuccess;
    const int64_t n_kt = (keys + NW * 32 - 1) / (NW * 32);
    const int64_t n_items = work_grid((int64_t)p.batch * p.Hkv, n_kt);
    if (n_items >= (1ll << 31)) return hipErrorInvalidValue;
    const int64_t resident = resident_workgroups<bwd_dkdv_kernel<D, NW, RT, PW>>(NW * 64);
    Params pk = p;
    pk.queue = p.queue + QUEUE_DKDV * N_XCD;
    hipLaunchKernelGGL((bwd_dkdv_kernel<D, NW, RT, PW>), dim3((unsigned)(n_items < resident ? n_items : resident)), dim3(NW * 64),
                       0, s, pk, (int)n_kt, (unsigned)(n_items / N_XCD));
    return hipGetLastError();
}

// Users with few query rows against long histories (see bwd_dkdv_resident_kernel): do the host-known bounds allow it,
// and are there enough (user, kv head) items to give every compute unit one?  (A workgroup walks all keys of its item
// by itself: with fewer items the key tiles of the streaming kernel spread better.)
template <int D>
bool few_rows_per_user(const Params& p) {
    const int64_t max_units = ((max_query_rows(p) + 31) / 32) * (p.Hq / p.Hkv);
    return D == 64 && !p.rt_len && !p.pointwise && max_units > 0 && max_units <= DkdvResident<D, 12>::MAX_UNITS &&
           max_lead_keys(p) >= 512 && (int64_t)p.batch * p.Hkv >= 256;
}

template <int D>
hipError_t launch_dkdv_resident(const Params& p, hipStream_t s) {
    constexpr int NW = 12;
    const int64_t n_items = work_grid((int64_t)p.batch * p.Hkv, 1);
    if (n_items >= (1ll << 31)) return hipErrorInvalidValue;
    const int64_t resident = resident_workgroups<bwd_dkdv_resident_kernel<D, NW>>(NW * 64);
    Params pk = p;
    pk.queue = p.queue + QUEUE_DKDV * N_XCD;
    hipLaunchKernelGGL((bwd_dkdv_resident_kernel<D, NW>), dim3((unsigned)(n_items < resident ? n_items : resident)), dim3(NW * 64),
                       0, s, pk, (unsigned)(n_items / N_XCD));
    return hipGetLastError();
}

template <int D, int NW>
hipError_t launch_dkdv(const Params& p, hipStream_t s) {
    if constexpr (D == 64) {
        if (few_rows_per_user<D>(p)) return launch_dkdv_resident<D>(p, s);
    }
    if (p.pointwise) return p.rt_len ? launch_dkdv_as<D, NW, true, true>(p, s) : launch_dkdv_as<D, NW, false, true>(p, s);
    return p.rt_len ? launch_dkdv_as<D, NW, true>(p, s) : launch_dkdv_as<D, NW, false>(p, s);
}

}  // namespace

hipError_t launch_bwd_bf16(const Params& p, hipStream_t s) {
    hipError_t e;
    // eight waves of one row block when the head group fills them, else four waves of two
    const bool wide = ((p.Hq / p.Hkv) % 8) == 0;
    timing_begin(MTFM_HTA_KERNEL_BWD_DQ, s);
    switch (p.d) {
        case 32: e = wide ? launch_dq<32, 2, 8>(p, s) : launch_dq<32, 2, 4>(p, s); break;
        case 64: e = wide ? launch_dq<64, 1, 8>(p, s) : launch_dq<64, 2, 4>(p, s); break;
        default: e = wide ? launch_dq<128, 1, 8>(p, s) : launch_dq<128, 1, 4>(p, s); break;
    }
    timing_end(MTFM_HTA_KERNEL_BWD_DQ, s);
    if (e != hipSuccess) return e;
    timing_begin(MTFM_HTA_KERNEL_BWD_DKDV, s);
    switch (p.d) {
        case 32: e = launch_dkdv<32, 4>(p, s); break;
        case 64: e = launch_dkdv<64, 4>(p, s); break;
        default: e = launch_dkdv<128, 4>(p, s); break;
    }
    timing_end(MTFM_HTA_KERNEL_BWD_DKDV, s);
    return e;
}

}  // namespace hta
