// bf16 backward of Hybrid Target Attention for gfx950, first launch: dQ (and the self-key blocks).
//
// Gradient of A = softmax_visible(scale Q K^T) V (the two attention equations of Section 3.2.2)
// with the probabilities recomputed from the saved logsumexp:
//   P = exp(scale S - lse),  dP = dO V^T,  dS = P o (dP - delta),  delta_i = <dO_i, O_i>,  dQ = scale dS K
// The whole backward pass is three pieces of work in two launches (see hta_bwd_bf16.hip); this file holds
//   1. bwd_self: the self-key terms of target rows' keys (rule 3: a target key is seen by its own row
//      only, so its dk/dv come from that row alone and are written here, final, in bf16).  Its blocks
//      are the last blocks of the dQ grid.
//   2. bwd_dq:   row-stationary, the forward kernel's decomposition: a wave keeps query rows (Q, dO, dQ) in
//      registers and streams the history K/V tiles through LDS.  S^T = K Q^T and dP^T = V dO^T have
//      the query row on the lane, so lse and delta are one register each and dS^T in accumulator layout
//      is directly the k-operand of dQ^T = K^T dS^T.  The self key of a target row is one extra term
//      in the epilogue.  dq is written once.  delta_i = <dO_i, O_i> is formed here, from the dO fragments
//      the wave holds anyway, and left (negated, with -lse/scale) in the workspace for the dK/dV launch.
// A translation unit of its own because it is compiled with another instruction scheduling strategy than the rest of
// the library (build.py: the strategy that favours instruction-level parallelism interleaves the dQ products of one
// row block with the weight arithmetic of the other, which the default, occupancy-driven strategy does not).
#include "../../include/mtfm_hta.h"
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

}  // namespace

hipError_t launch_bwd_dq_bf16(const Params& p, hipStream_t s) {
    // eight waves of one row block when the head group fills them, else four waves of two
    const bool wide = ((p.Hq / p.Hkv) % 8) == 0;
    switch (p.d) {
        case 32: return wide ? launch_dq<32, 2, 8>(p, s) : launch_dq<32, 2, 4>(p, s);
        case 64: return wide ? launch_dq<64, 1, 8>(p, s) : launch_dq<64, 2, 4>(p, s);
        default: return wide ? launch_dq<128, 1, 8>(p, s) : launch_dq<128, 1, 4>(p, s);
    }
}

}  // namespace hta
