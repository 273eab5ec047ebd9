// The dK/dV pass of the bf16 backward (gfx950): kernel templates and their launchers, included by the translation
// units that instantiate them (hta_bwd_bf16.hip: all but one; hta_bwd_dkdv128_bf16.hip: the head_dim 128 softmax kernel,
// compiled with another instruction scheduling strategy, see build.py).
//
//   bwd_dkdv: key-stationary: a wave owns 32 history keys (K, V fragments and the dK, dV accumulators
//      stay in registers for the whole kernel), the workgroup streams (head, 32-row block) tiles of Q
//      and dO through LDS, shared by its waves.  S = Q K^T and dP = dO V^T have the key on the lane, so
//      P and dS in accumulator layout are directly the k-operand of dV = P^T dO and dK = dS^T Q.
//      dk/dv of history keys are written once.
#pragma once
#include "../../include/mtfm_hta.h"
#include "hta_common.h"
#include "hta_mfma.h"
#include "hta_tiles.h"

namespace hta {
namespace {

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
}  // namespace hta
