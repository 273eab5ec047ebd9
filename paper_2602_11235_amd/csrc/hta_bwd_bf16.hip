// bf16 backward kernels of Hybrid Target Attention for gfx950.
//
// Gradient of A = softmax_visible(scale Q K^T) V (the two attention equations of Section 3.2.2)
// with the probabilities recomputed from the saved logsumexp:
//   P = exp(scale S - lse),  dP = dO V^T,  dS = P o (dP - delta),  delta_i = <dO_i, O_i>
//   dV = P^T dO,  dK = scale dS^T Q  (both summed over the query heads of the kv group),  dQ = scale dS K
//
// Three kernels:
//   1. bwd_pre:  delta for every (row, head); the self-key terms of target rows (rule 3: a target
//      key is seen by its own row only, so its dk/dv come from that row alone and are written here,
//      final, in bf16); and the float32 dq accumulator initialised to the self term (zero for
//      history rows).
//   2. bwd_main: one workgroup per (user, kv head, tile of BN history keys).  K/V tile in LDS,
//      shared by all query heads of the group.  Each wave walks over (head, 32-row block) units:
//      five 32x32x16 bf16 MFMA products per unit and 32-key sub-block, dK/dV kept in registers for
//      the whole walk, dQ added to the float32 accumulator with atomics (it is a sum over key
//      tiles, i.e. over workgroups).  Only history keys are ever visited: target x target and
//      history-row x target-key tiles do not exist under the hybrid mask.
//   3. bwd_post: dq accumulator -> bf16.
//
// MFMA operand choreography (see hta_mfma.h for the lane layouts): S = Q K^T and dP = dO V^T are
// computed with the query rows on the accumulator *registers* and the keys on the lanes, so P and
// dS are directly the k-operand of the products that contract over rows (dV, dK).  dQ contracts
// over keys, which sit on lanes, so dS takes one wave-private round trip through LDS.  Every
// transposed operand (Q^T, dO^T, K^T, dS^T) is produced by the LDS transpose read from a row-major
// tile; nothing is transposed when staged.
#include "../../include/mtfm_hta.h"
#include "hta_common.h"
#include "hta_mfma.h"

namespace hta {
namespace {

__device__ inline float group_sum(float x, int width) {  // sum over aligned groups of `width` lanes
    for (int o = width >> 1; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// ---------------------------------------------------------------------------------------- pre
// One group of D/8 lanes per (query row, kv head); the group walks the r query heads of the kv head.
template <int D>
__global__ __launch_bounds__(256) void bwd_pre_kernel(Params p) {
    constexpr int LPR = D / 8;           // lanes per item, 8 elements (16 bytes) each
    constexpr int IPB = 256 / LPR;       // items per block
    const int b = blockIdx.z;
    const int L = p.hist_len[b], T = p.n_targets[b];
    const int n_rows = p.layer == 0 ? L + T : T;
    const int r = p.Hq / p.Hkv;
    const int item = blockIdx.x * IPB + threadIdx.x / LPR;  // (row, g) flattened, g fastest
    const int sub = threadIdx.x % LPR;
    const int row = item / p.Hkv, g = item % p.Hkv;
    if (row >= n_rows) return;  // whole lane groups leave together; group_sum only talks inside a group
    const int64_t q_row = (int64_t)p.q_off[b] + row;
    const int tok = (p.layer == 0 ? 0 : L) + row;
    const bool is_target = tok >= L;
    const __bf16* qg = (const __bf16*)p.q;
    const __bf16* dog = (const __bf16*)p.dout;
    const __bf16* og = (const __bf16*)p.out;
    float kself[8], vself[8], dk_t[8], dv_t[8];
    int64_t kv_off = 0;
    if (is_target) {
        kv_off = (((int64_t)p.kv_off[b] + tok) * p.Hkv + g) * D + sub * 8;
        const bf16x8 kk = *(const bf16x8*)((const __bf16*)p.k + kv_off);
        const bf16x8 vv = *(const bf16x8*)((const __bf16*)p.v + kv_off);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            kself[j] = (float)kk[j];
            vself[j] = (float)vv[j];
            dk_t[j] = 0.f;
            dv_t[j] = 0.f;
        }
    }
    for (int hh = 0; hh < r; hh++) {
        const int h = g * r + hh;
        const int64_t off = (q_row * p.Hq + h) * D + sub * 8;
        const bf16x8 dov = *(const bf16x8*)(dog + off);
        const bf16x8 ov = *(const bf16x8*)(og + off);
        float dof[8], part = 0.f;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            dof[j] = (float)dov[j];
            part = fmaf(dof[j], (float)ov[j], part);
        }
        const float delta = group_sum(part, LPR);
        if (sub == 0) p.delta[(int64_t)h * p.total_q + q_row] = delta;
        float dq0[8];
#pragma unroll
        for (int j = 0; j < 8; j++) dq0[j] = 0.f;
        if (is_target) {
            const bf16x8 qv = *(const bf16x8*)(qg + off);
            float qf[8], sp = 0.f, dpp = 0.f;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                qf[j] = (float)qv[j];
                sp = fmaf(qf[j], kself[j], sp);
                dpp = fmaf(dof[j], vself[j], dpp);
            }
            const float s = group_sum(sp, LPR) * p.scale;
            const float dp = group_sum(dpp, LPR);
            const float pw = __expf(s - p.lse[(int64_t)h * p.total_q + q_row]);
            const float ds = pw * (dp - delta) * p.scale;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                dq0[j] = ds * kself[j];
                dk_t[j] = fmaf(ds, qf[j], dk_t[j]);
                dv_t[j] = fmaf(pw, dof[j], dv_t[j]);
            }
        }
        float* dqa = p.dq_acc + off;
        *(float4*)dqa = make_float4(dq0[0], dq0[1], dq0[2], dq0[3]);
        *(float4*)(dqa + 4) = make_float4(dq0[4], dq0[5], dq0[6], dq0[7]);
    }
    if (is_target) {
        bf16x8 dk8, dv8;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            dk8[j] = (__bf16)dk_t[j];
            dv8[j] = (__bf16)dv_t[j];
        }
        *(bf16x8*)((__bf16*)p.dk + kv_off) = dk8;
        *(bf16x8*)((__bf16*)p.dv + kv_off) = dv8;
    }
}

// ---------------------------------------------------------------------------------------- post
__global__ __launch_bounds__(256) void bwd_post_kernel(const float* __restrict__ acc, __bf16* __restrict__ dq, int64_t n8) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n8; i += stride) {
        const float4 a = *(const float4*)(acc + i * 8);
        const float4 c = *(const float4*)(acc + i * 8 + 4);
        bf16x8 o;
        o[0] = (__bf16)a.x; o[1] = (__bf16)a.y; o[2] = (__bf16)a.z; o[3] = (__bf16)a.w;
        o[4] = (__bf16)c.x; o[5] = (__bf16)c.y; o[6] = (__bf16)c.z; o[7] = (__bf16)c.w;
        *(bf16x8*)(dq + i * 8) = o;
    }
}

// ---------------------------------------------------------------------------------------- main
template <int D, int BN, int NW>
struct BwdSmem {
    static constexpr int KS = D + 8;       // K/V row pitch (elements)
    static constexpr int QS = D + 8;       // wave-private Q/dO row pitch
    static constexpr int SS = 32 + 8;      // wave-private dS [key][row] pitch
    static constexpr int KV_ELEMS = 2 * BN * KS;
    static constexpr int WAVE_ELEMS = 2 * 32 * QS + 32 * SS;
    static constexpr size_t WAVE_BYTES = (size_t)WAVE_ELEMS * 2;
    static constexpr size_t RED_BYTES = (size_t)BN * D * 4;   // float32 [key][d] reduction buffer, aliased on the wave regions
    static constexpr size_t BYTES = (size_t)KV_ELEMS * 2 + (NW * WAVE_BYTES > RED_BYTES ? NW * WAVE_BYTES : RED_BYTES);
};

template <int D, int BN, int NW>
__global__ __launch_bounds__(NW * 64) void bwd_main_kernel(Params p) {
    using SM = BwdSmem<D, BN, NW>;
    constexpr int NT = NW * 64;
    constexpr int KS = SM::KS, QS = SM::QS, SS = SM::SS;
    constexpr int CPR = D / 8, NCH = BN * CPR;
    constexpr int NKS = D / 16, NDB = D / 32, NKB = BN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __bf16* Ks = (__bf16*)smem_raw;
    __bf16* Vs = Ks + BN * KS;
    unsigned char* wave_base = smem_raw + (size_t)SM::KV_ELEMS * 2;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    const int b = blockIdx.z, g = blockIdx.y, kt = blockIdx.x;
    const int L = p.hist_len[b], T = p.n_targets[b];
    if (kt * BN >= L) return;  // uniform: this key tile does not exist for the user
    const int n_rows = p.layer == 0 ? L + T : T;
    const int r = p.Hq / p.Hkv;
    const int64_t q_base = p.q_off[b], kv_base = p.kv_off[b];
    const __bf16* qg = (const __bf16*)p.q;
    const __bf16* dog = (const __bf16*)p.dout;
    const float c2 = p.scale * LOG2E;
    const int key0 = kt * BN;

    // stage the K/V tile (keys past the history are zero-filled; their P and dS are forced to 0)
    for (int c = tid; c < NCH; c += NT) {
        const int key = c / CPR, dc = c % CPR;
        uint4 kk = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
        if (key0 + key < L) {
            const int64_t off = ((kv_base + key0 + key) * p.Hkv + g) * D + dc * 8;
            kk = *(const uint4*)((const __bf16*)p.k + off);
            vv = *(const uint4*)((const __bf16*)p.v + off);
        }
        *(uint4*)(Ks + key * KS + dc * 8) = kk;
        *(uint4*)(Vs + key * KS + dc * 8) = vv;
    }
    __syncthreads();

    __bf16* Qs = (__bf16*)(wave_base + wave * SM::WAVE_BYTES);
    __bf16* dOs = Qs + 32 * QS;
    __bf16* dSs = dOs + 32 * QS;

    floatx16 dK[NKB][NDB], dV[NKB][NDB];  // [key m (registers)][d n (lanes)]
#pragma unroll
    for (int kb = 0; kb < NKB; kb++)
#pragma unroll
        for (int db = 0; db < NDB; db++)
#pragma unroll
            for (int v = 0; v < 16; v++) {
                dK[kb][db][v] = 0.f;
                dV[kb][db][v] = 0.f;
            }
    const bool ragged_keys = key0 + BN > L;
    const int n_rb = (n_rows + 31) / 32;
    const int n_units = n_rb * r;
    const int dhalf = (lane >> 4) & 1;

    for (int u = wave; u < n_units; u += NW) {
        const int rb = u / r, h = g * r + u % r;
        const int row0 = rb * 32;
        // Q and dO rows of the unit: natural fragments (lane = row, 8 consecutive d per k-step) straight from
        // global memory, and a copy in the wave's LDS region for the transposed reads
        bf16x8 qf[NKS], dof[NKS];
        {
            int row = row0 + l32;
            row = row < n_rows ? row : n_rows - 1;
            const int64_t off = ((q_base + row) * p.Hq + h) * D + 8 * hf;
#pragma unroll
            for (int ks = 0; ks < NKS; ks++) {
                qf[ks] = *(const bf16x8*)(qg + off + ks * 16);
                dof[ks] = *(const bf16x8*)(dog + off + ks * 16);
            }
#pragma unroll
            for (int ks = 0; ks < NKS; ks++) {
                *(bf16x8*)(Qs + l32 * QS + ks * 16 + 8 * hf) = qf[ks];
                *(bf16x8*)(dOs + l32 * QS + ks * 16 + 8 * hf) = dof[ks];
            }
        }
        // per accumulator register: lse (log2 domain) and delta of its row; rows past the end get lse = +inf => P = 0
        float lse2[16], dl[16];
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int row = row0 + 8 * (v / 4) + 4 * hf + (v % 4);
            const bool live = row < n_rows;
            const int64_t idx = (int64_t)h * p.total_q + q_base + (live ? row : n_rows - 1);
            lse2[v] = live ? p.lse[idx] * LOG2E : INFINITY;
            dl[v] = p.delta[idx];
        }
        floatx16 dQ[NDB];  // [row m (registers)][d n (lanes)]
#pragma unroll
        for (int db = 0; db < NDB; db++)
#pragma unroll
            for (int v = 0; v < 16; v++) dQ[db][v] = 0.f;

#pragma unroll
        for (int kb = 0; kb < NKB; kb++) {
            floatx16 S, dP;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                S[v] = 0.f;
                dP[v] = 0.f;
            }
#pragma unroll
            for (int ks = 0; ks < NKS; ks++) {
                const bf16x8 kf = *(const bf16x8*)(Ks + (kb * 32 + l32) * KS + ks * 16 + 8 * hf);
                const bf16x8 vf = *(const bf16x8*)(Vs + (kb * 32 + l32) * KS + ks * 16 + 8 * hf);
                S = mfma32(qf[ks], kf, S);      // S[row][key]
                dP = mfma32(dof[ks], vf, dP);   // dP[row][key]
            }
            const bool key_dead = ragged_keys && (key0 + kb * 32 + l32 >= L);
            bf16x8 pb[2], dsb[2];
#pragma unroll
            for (int v = 0; v < 16; v++) {
                float pw = fast_exp2(fmaf(S[v], c2, -lse2[v]));
                pw = key_dead ? 0.f : pw;
                const float ds = pw * (dP[v] - dl[v]);
                pb[v / 8][v % 8] = (__bf16)pw;
                dsb[v / 8][v % 8] = (__bf16)ds;
            }
            // dS^T to the wave's LDS region as [key][row]: this lane owns key l32 and rows 8j+4hf..+3
#pragma unroll
            for (int j = 0; j < 4; j++) {
                bf16x4 w;
                w[0] = dsb[j / 2][4 * (j % 2) + 0];
                w[1] = dsb[j / 2][4 * (j % 2) + 1];
                w[2] = dsb[j / 2][4 * (j % 2) + 2];
                w[3] = dsb[j / 2][4 * (j % 2) + 3];
                *(bf16x4*)(dSs + l32 * SS + 8 * j + 4 * hf) = w;
            }
            // dV[key][d] += P^T[key][row] dO[row][d];  dK[key][d] += dS^T[key][row] Q[row][d]
#pragma unroll
            for (int db = 0; db < NDB; db++)
#pragma unroll
                for (int s2 = 0; s2 < 2; s2++) {
                    const bf16x8 dot = lds_read_tr_8(dOs, QS, 16 * s2 + 4 * hf, db * 32 + 16 * dhalf, lane);
                    const bf16x8 qt = lds_read_tr_8(Qs, QS, 16 * s2 + 4 * hf, db * 32 + 16 * dhalf, lane);
                    dV[kb][db] = mfma32(pb[s2], dot, dV[kb][db]);
                    dK[kb][db] = mfma32(dsb[s2], qt, dK[kb][db]);
                }
            // dQ[row][d] += dS[row][key] K[key][d]
#pragma unroll
            for (int s2 = 0; s2 < 2; s2++) {
                const bf16x8 dst = lds_read_tr_8(dSs, SS, 16 * s2 + 4 * hf, 16 * dhalf, lane);
#pragma unroll
                for (int db = 0; db < NDB; db++) {
                    const bf16x8 ktf = lds_read_tr_8(Ks + kb * 32 * KS, KS, 16 * s2 + 4 * hf, db * 32 + 16 * dhalf, lane);
                    dQ[db] = mfma32(dst, ktf, dQ[db]);
                }
            }
        }
        // dQ partial of this key tile -> float32 accumulator (lanes cover 32 consecutive d: coalesced atomics)
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int row = row0 + 8 * (v / 4) + 4 * hf + (v % 4);
            if (row < n_rows) {
                float* dst = p.dq_acc + ((q_base + row) * p.Hq + h) * D + l32;
#pragma unroll
                for (int db = 0; db < NDB; db++) atomicAdd(dst + db * 32, dQ[db][v] * p.scale);
            }
        }
    }

    // sum dK / dV over the waves through LDS, then write bf16 rows of the history keys
    __syncthreads();  // all waves are done with their private regions
    float* red = (float*)wave_base;
#pragma unroll 1
    for (int which = 0; which < 2; which++) {
        for (int i = tid; i < BN * D; i += NT) red[i] = 0.f;
        __syncthreads();
#pragma unroll
        for (int kb = 0; kb < NKB; kb++)
#pragma unroll
            for (int db = 0; db < NDB; db++)
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    const int key = kb * 32 + 8 * (v / 4) + 4 * hf + (v % 4);
                    const float val = which == 0 ? dK[kb][db][v] * p.scale : dV[kb][db][v];
                    atomicAdd(red + key * D + db * 32 + l32, val);
                }
        __syncthreads();
        __bf16* dst = (__bf16*)(which == 0 ? p.dk : p.dv);
        for (int c = tid; c < NCH; c += NT) {
            const int key = c / CPR, dc = c % CPR;
            if (key0 + key < L) {
                bf16x8 o;
#pragma unroll
                for (int j = 0; j < 8; j++) o[j] = (__bf16)red[key * D + dc * 8 + j];
                *(bf16x8*)(dst + ((kv_base + key0 + key) * p.Hkv + g) * D + dc * 8) = o;
            }
        }
        __syncthreads();
    }
}

template <int D, int BN, int NW>
hipError_t launch_main(const Params& p, hipStream_t s) {
    using SM = BwdSmem<D, BN, NW>;
    if (p.max_hist <= 0) return hipSuccess;
    static bool configured = false;  // raising the dynamic LDS limit is a per-function, process-wide setting
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)bwd_main_kernel<D, BN, NW>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)SM::BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    dim3 grid((unsigned)((p.max_hist + BN - 1) / BN), (unsigned)p.Hkv, (unsigned)p.batch);
    hipLaunchKernelGGL((bwd_main_kernel<D, BN, NW>), grid, dim3(NW * 64), SM::BYTES, s, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_pre(const Params& p, hipStream_t s) {
    const int64_t rows = max_query_rows(p);
    if (rows <= 0) return hipSuccess;
    constexpr int IPB = 256 / (D / 8);
    const int64_t items = rows * p.Hkv;
    dim3 grid((unsigned)((items + IPB - 1) / IPB), 1, (unsigned)p.batch);
    hipLaunchKernelGGL(bwd_pre_kernel<D>, grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_bf16(const Params& p, hipStream_t s) {
    hipError_t e;
    timing_begin(MTFM_HTA_KERNEL_BWD_PRE, s);
    switch (p.d) {
        case 32: e = launch_pre<32>(p, s); break;
        case 64: e = launch_pre<64>(p, s); break;
        case 128: e = launch_pre<128>(p, s); break;
        default: e = hipErrorInvalidValue;
    }
    timing_end(MTFM_HTA_KERNEL_BWD_PRE, s);
    if (e != hipSuccess) return e;
    timing_begin(MTFM_HTA_KERNEL_BWD_MAIN, s);
    switch (p.d) {
        case 32: e = launch_main<32, 64, 4>(p, s); break;
        case 64: e = launch_main<64, 64, 4>(p, s); break;
        default: e = launch_main<128, 32, 4>(p, s); break;
    }
    timing_end(MTFM_HTA_KERNEL_BWD_MAIN, s);
    if (e != hipSuccess) return e;
    const int64_t n8 = p.total_q * p.Hq * p.d / 8;
    if (n8 > 0) {
        int64_t blocks = (n8 + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        timing_begin(MTFM_HTA_KERNEL_BWD_POST, s);
        hipLaunchKernelGGL(bwd_post_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p.dq_acc, (__bf16*)p.dq, n8);
        e = hipGetLastError();
        timing_end(MTFM_HTA_KERNEL_BWD_POST, s);
    }
    return e;
}

}  // namespace hta
