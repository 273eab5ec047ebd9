// Fused group layer normalization (Section 3.2.2, the fused operator of Section 3.3.2) for gfx950: forward,
// backward and the C ABI of include/mtfm_gln.h.
//
// The work is bound by HBM: a token is read once and written once, its arithmetic is a few dozen flops per
// element.  One wave owns a token at a time: lane l holds features [8 l, 8 l + 8) of every 512-feature chunk
// (16-byte loads of bf16), the two row statistics are wave reductions in registers, and nothing is gathered or
// scattered -- a token picks its group's parameter row out of LDS, where all rows are staged once per workgroup.
// Workgroups are persistent (a fixed grid strides over the tokens), which also bounds the number of partial
// parameter gradients of the backward pass: each workgroup accumulates dgamma / dbeta of all groups in LDS
// (float atomic adds) and writes its share once; a second kernel sums the shares in a fixed order.
#include "../../include/mtfm_gln.h"
#include "hta_common.h"

#include <hip/hip_runtime.h>

namespace gln {

constexpr int THREADS = 512;
constexpr int WAVES = THREADS / 64;
constexpr int MAX_BLOCKS = 512;   // workgroups of a launch, and shares of dgamma / dbeta in the workspace
constexpr int CHUNK = 512;        // features a wave covers per pass: 64 lanes x 8
constexpr int MAX_CHUNKS = 4;     // d_model <= 2048
constexpr int MAX_TABLE = 8192;   // n_groups x padded row length, in floats
constexpr int MAX_GROUPS = MAX_TABLE / CHUNK;
constexpr int REDUCE_SLICES = 16, REDUCE_COLS = 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct Args {
    const void *x, *gate, *dy;
    const int32_t* group_id;
    const float *gamma, *beta, *mean_in, *rstd_in;
    void *y, *dx, *dgate;
    float *mean, *rstd, *partials;
    int64_t n;
    int32_t d, n_groups, row;  // row = d rounded up to whole chunks: the stride of a group's row in LDS
    int32_t span;              // backward: tokens a wave takes per pass, at most 64 (a workgroup: WAVES times that)
    float eps;
};

// eight consecutive features as they lie in memory; converted where they are used, so that tokens waiting for
// their turn occupy half the registers in bf16
template <typename T>
struct Raw;
template <>
struct Raw<__bf16> {
    bf16x8 v;
    __device__ void load(const __bf16* p) { v = __builtin_nontemporal_load((const bf16x8*)p); }
    __device__ float operator[](int j) const { return (float)v[j]; }
};
template <>
struct Raw<float> {
    floatx4 lo, hi;
    __device__ void load(const float* p) { lo = *(const floatx4*)p, hi = *(const floatx4*)(p + 4); }
    __device__ float operator[](int j) const { return j < 4 ? lo[j] : hi[j - 4]; }
};

__device__ inline void load8(const __bf16* p, float (&f)[8]) {
    const bf16x8 v = __builtin_nontemporal_load((const bf16x8*)p);
#pragma unroll
    for (int j = 0; j < 8; j++) f[j] = (float)v[j];
}
__device__ inline void load8(const float* p, float (&f)[8]) {
    const floatx4 a = *(const floatx4*)p, b = *(const floatx4*)(p + 4);
#pragma unroll
    for (int j = 0; j < 4; j++) f[j] = a[j], f[4 + j] = b[j];
}
__device__ inline void store8(__bf16* p, const float (&f)[8]) {
    bf16x8 v;
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = (__bf16)f[j];  // round to nearest even
    __builtin_nontemporal_store(v, (bf16x8*)p);  // written once, not read again by this kernel
}
__device__ inline void store8(float* p, const float (&f)[8]) {
    floatx4 a, b;
#pragma unroll
    for (int j = 0; j < 4; j++) a[j] = f[j], b[j] = f[4 + j];
    *(floatx4*)p = a;
    *(floatx4*)(p + 4) = b;
}

template <int CTRL>
__device__ inline float dpp(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
// sum over the 64 lanes in a fixed order, the same value in every lane: exchanges inside the 16-lane rows
// (lane ^ 1, lane ^ 2, mirror of each half row, mirror of the row), then the four row sums
__device__ inline float wave_sum(float v) {
    v += dpp<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp<0x141>(v);  // row_half_mirror
    v += dpp<0x140>(v);  // row_mirror
    const int u = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(u, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(u, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(u, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(u, 48));
    return (r0 + r1) + (r2 + r3);
}

// Where feature e of a parameter row lies in LDS.  A lane reads its 8 features of a chunk as two 16-byte words:
// the first words of the 64 lanes are contiguous, then the second words, so neither read has a bank conflict.
__device__ inline int quad_slot(int e) {
    const int r = e & (CHUNK - 1);
    return (e - r) + ((r >> 2) & 1) * 256 + (r >> 3) * 4 + (r & 3);
}
// Where the accumulator of feature e lies: feature j of lane l at word j * 64 + l of the chunk, so the 64
// atomic adds of one instruction fall into 64 different banks.
__device__ inline int word_slot(int e) {
    const int r = e & (CHUNK - 1);
    return (e - r) + (r & 7) * 64 + (r >> 3);
}

__device__ inline void stage_rows(float* table, const float* src, int n_groups, int d, int row) {
    for (int i = threadIdx.x * 4; i < n_groups * d; i += THREADS * 4) {
        const int g = i / d, e = i - g * d;
        *(floatx4*)&table[g * row + quad_slot(e)] = *(const floatx4*)&src[i];
    }
}

__device__ inline void read_row8(const float* table_row, int c, int lane, float (&f)[8]) {
    const floatx4 a = *(const floatx4*)&table_row[c * CHUNK + lane * 4];
    const floatx4 b = *(const floatx4*)&table_row[c * CHUNK + 256 + lane * 4];
#pragma unroll
    for (int j = 0; j < 4; j++) f[j] = a[j], f[4 + j] = b[j];
}

__device__ inline int group_of(const Args& a, int64_t t) {
    const int g = __builtin_amdgcn_readfirstlane(a.group_id[t]);
    return g < 0 ? 0 : (g >= a.n_groups ? a.n_groups - 1 : g);
}

// TPW tokens per wave and iteration: their loads are all issued before the first is used
template <typename T, int CPL, bool GATED>
__global__ __launch_bounds__(THREADS, CPL <= 2 ? 4 : 2) void fwd_kernel(const Args a) {
    constexpr int TPW = CPL == 1 ? 2 : 1;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* gamma_s = smem;
    float* beta_s = smem + a.n_groups * a.row;
    stage_rows(gamma_s, a.gamma, a.n_groups, a.d, a.row);
    stage_rows(beta_s, a.beta, a.n_groups, a.d, a.row);
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d = a.d;
    const float inv_d = 1.f / (float)d;
    const T* xg = (const T*)a.x;
    const T* ug = (const T*)a.gate;
    T* yg = (T*)a.y;
    const int64_t stride = (int64_t)gridDim.x * WAVES * TPW;
    for (int64_t t0 = ((int64_t)blockIdx.x * WAVES + wave) * TPW; t0 < a.n; t0 += stride) {
        float xv[TPW][CPL][8], uv[TPW][CPL][8];
#pragma unroll
        for (int k = 0; k < TPW; k++) {
            const int64_t t = t0 + k;
#pragma unroll
            for (int c = 0; c < CPL; c++) {
                const int col = (c * 64 + lane) * 8;
                if (t < a.n && col < d) {
                    load8(xg + t * d + col, xv[k][c]);
                    if (GATED) load8(ug + t * d + col, uv[k][c]);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; j++) xv[k][c][j] = 0.f;
                }
            }
        }
#pragma unroll
        for (int k = 0; k < TPW; k++) {
            const int64_t t = t0 + k;
            if (t >= a.n) break;
            float s = 0.f;
#pragma unroll
            for (int c = 0; c < CPL; c++)
#pragma unroll
                for (int j = 0; j < 8; j++) s += xv[k][c][j];
            // Centre on a first mean m, then correct it by the mean of the centred values: x - m is exact for a
            // token whose spread is small against its offset, where the rounding of m itself would dominate.
            const float m = wave_sum(s) * inv_d;
            float q = 0.f, r = 0.f;
#pragma unroll
            for (int c = 0; c < CPL; c++) {
                if ((c * 64 + lane) * 8 < d) {
#pragma unroll
                    for (int j = 0; j < 8; j++) {
                        xv[k][c][j] -= m;
                        r += xv[k][c][j];
                        q += xv[k][c][j] * xv[k][c][j];
                    }
                }
            }
            const float delta = wave_sum(r) * inv_d;
            const float var = fmaxf(wave_sum(q) * inv_d - delta * delta, 0.f);
            const float mean = m + delta;
            const float rstd = 1.f / sqrtf(var + a.eps);
            const int g = group_of(a, t);
#pragma unroll
            for (int c = 0; c < CPL; c++) {
                const int col = (c * 64 + lane) * 8;
                if (col < d) {
                    float gm[8], bt[8], out[8];
                    read_row8(gamma_s + g * a.row, c, lane, gm);
                    read_row8(beta_s + g * a.row, c, lane, bt);
#pragma unroll
                    for (int j = 0; j < 8; j++) {
                        out[j] = gm[j] * ((xv[k][c][j] - delta) * rstd) + bt[j];
                        if (GATED) out[j] *= uv[k][c][j];
                    }
                    store8(yg + t * d + col, out);
                }
            }
            if (lane == 0) {
                if (a.mean) a.mean[t] = mean;
                if (a.rstd) a.rstd[t] = rstd;
            }
        }
    }
}

// Backward.  A wave takes up to 64 tokens at a time (lane l holds the group and position of the l-th of them)
// and works through them group by group: the tokens of one group add their dz (.) xhat and dz into registers, and
// only when the group is done do these go to the workgroup's accumulators in LDS -- a few atomic adds per span
// instead of sixteen per token.
template <typename T, int CPL, bool GATED>
__global__ __launch_bounds__(THREADS, CPL == 1 ? 4 : 2) void bwd_kernel(const Args a) {
    constexpr int TPW = CPL == 1 && sizeof(T) == 2 ? 2 : 1;  // tokens in flight per wave
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int table = a.n_groups * a.row;
    float* gamma_s = smem;
    float* dgamma_s = smem + table;
    float* dbeta_s = smem + 2 * table;
    float* beta_s = smem + 3 * table;  // present only with a gate
    stage_rows(gamma_s, a.gamma, a.n_groups, a.d, a.row);
    if (GATED) stage_rows(beta_s, a.beta, a.n_groups, a.d, a.row);
    for (int i = threadIdx.x; i < 2 * table; i += THREADS) dgamma_s[i] = 0.f;
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d = a.d;
    const float inv_d = 1.f / (float)d;
    const T* dyg = (const T*)a.dy;
    const T* xg = (const T*)a.x;
    const T* ug = (const T*)a.gate;
    T* dxg = (T*)a.dx;
    T* dug = (T*)a.dgate;
    // A workgroup takes a span of up to 512 consecutive tokens per pass and orders it by group (a counting sort of
    // the ids in LDS); each wave then takes an equal share of the ordered span, so it meets only the few groups
    // its share straddles, however skewed the group sizes are.
    __shared__ int sorted_s[THREADS];           // (group << 16) | offset of the token in the span
    __shared__ int counts_s[WAVES][MAX_GROUPS];  // tokens of each group among a wave's 64 candidates
    const int block_span = a.span * WAVES;
    for (int64_t base = (int64_t)blockIdx.x * block_span; base < a.n; base += (int64_t)gridDim.x * block_span) {
        const int live = (int)(a.n - base < block_span ? a.n - base : block_span);
        int g_me = -1;
        if ((int)threadIdx.x < live) {
            const int g = a.group_id[base + threadIdx.x];
            g_me = g < 0 ? 0 : (g >= a.n_groups ? a.n_groups - 1 : g);
        }
        int rank = 0;
        for (int g = 0; g < a.n_groups; g++) {
            const uint64_t m = __ballot(g_me == g);
            if (g_me == g) rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
            if (lane == 0) counts_s[wave][g] = __builtin_popcountll(m);
        }
        __syncthreads();
        if (g_me >= 0) {
            int pos = rank;
            for (int g = 0; g < g_me; g++)
                for (int w = 0; w < WAVES; w++) pos += counts_s[w][g];
            for (int w = 0; w < wave; w++) pos += counts_s[w][g_me];
            sorted_s[pos] = (g_me << 16) | (int)threadIdx.x;
        }
        __syncthreads();
        const int per_wave = (live + WAVES - 1) / WAVES;
        int g_lane = -1, off_lane = 0;
        if (lane < per_wave && wave * per_wave + lane < live) {
            const int e = sorted_s[wave * per_wave + lane];
            g_lane = e >> 16, off_lane = e & 0xFFFF;
        }
        uint64_t todo = __ballot(g_lane >= 0);
        while (todo) {
            const int g = __builtin_amdgcn_readlane(g_lane, __builtin_ctzll(todo));
            uint64_t members = __ballot(g_lane == g);
            todo &= ~members;
            float acc_g[CPL][8], acc_b[CPL][8];
#pragma unroll
            for (int c = 0; c < CPL; c++)
#pragma unroll
                for (int j = 0; j < 8; j++) acc_g[c][j] = 0.f, acc_b[c][j] = 0.f;
            while (members) {
                int64_t tok[TPW];
#pragma unroll
                for (int k = 0; k < TPW; k++) {
                    tok[k] = members ? base + __builtin_amdgcn_readlane(off_lane, __builtin_ctzll(members)) : -1;
                    members &= members - 1;  // stays 0 once empty
                }
                Raw<T> gv[TPW][CPL], xv[TPW][CPL], uv[TPW][CPL];
                float mean[TPW], rstd[TPW];
#pragma unroll
                for (int k = 0; k < TPW; k++) {
                    const int64_t t = tok[k];
                    if (t >= 0) {
                        mean[k] = a.mean_in[t];
                        rstd[k] = a.rstd_in[t];
                    }
#pragma unroll
                    for (int c = 0; c < CPL; c++) {
                        const int col = (c * 64 + lane) * 8;
                        if (t >= 0 && col < d) {
                            gv[k][c].load(dyg + t * d + col);
                            xv[k][c].load(xg + t * d + col);
                            if (GATED) uv[k][c].load(ug + t * d + col);
                        }
                    }
                }
#pragma unroll
                for (int k = 0; k < TPW; k++) {
                    const int64_t t = tok[k];
                    if (t < 0) break;
                    float s1 = 0.f, s2 = 0.f;
                    float w[CPL][8], xh[CPL][8];
#pragma unroll
                    for (int c = 0; c < CPL; c++) {
                        const int col = (c * 64 + lane) * 8;
                        if (col < d) {
                            float gm[8];
                            read_row8(gamma_s + g * a.row, c, lane, gm);
#pragma unroll
                            for (int j = 0; j < 8; j++) {
                                xh[c][j] = (xv[k][c][j] - mean[k]) * rstd[k];
                                const float dz = GATED ? gv[k][c][j] * uv[k][c][j] : gv[k][c][j];
                                w[c][j] = dz * gm[j];
                                s1 += w[c][j];
                                s2 += w[c][j] * xh[c][j];
                                acc_g[c][j] += dz * xh[c][j];
                                acc_b[c][j] += dz;
                            }
                            if (GATED) {
                                float bt[8], du[8];
                                read_row8(beta_s + g * a.row, c, lane, bt);
#pragma unroll
                                for (int j = 0; j < 8; j++) du[j] = gv[k][c][j] * (gm[j] * xh[c][j] + bt[j]);
                                store8(dug + t * d + col, du);
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < 8; j++) w[c][j] = 0.f, xh[c][j] = 0.f;
                        }
                    }
                    s1 = wave_sum(s1) * inv_d;
                    s2 = wave_sum(s2) * inv_d;
#pragma unroll
                    for (int c = 0; c < CPL; c++) {
                        const int col = (c * 64 + lane) * 8;
                        if (col < d) {
                            float out[8];
#pragma unroll
                            for (int j = 0; j < 8; j++) out[j] = rstd[k] * (w[c][j] - s1 - xh[c][j] * s2);
                            store8(dxg + t * d + col, out);
                        }
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < CPL; c++) {
                if ((c * 64 + lane) * 8 < d) {
                    float* slot_g = dgamma_s + g * a.row + c * CHUNK + lane;
                    float* slot_b = dbeta_s + g * a.row + c * CHUNK + lane;
#pragma unroll
                    for (int j = 0; j < 8; j++) {
                        atomicAdd(slot_g + j * 64, acc_g[c][j]);
                        atomicAdd(slot_b + j * 64, acc_b[c][j]);
                    }
                }
            }
        }
    }
    __syncthreads();
    // this workgroup's share, features in their natural order: [dgamma | dbeta][n_groups][d]
    const int gd = a.n_groups * d;
    float* share = a.partials + (size_t)blockIdx.x * 2 * gd;
    for (int i = threadIdx.x; i < gd; i += THREADS) {
        const int g = i / d, e = i - g * d;
        share[i] = dgamma_s[g * a.row + word_slot(e)];
        share[gd + i] = dbeta_s[g * a.row + word_slot(e)];
    }
}

// dgamma | dbeta = the sum of the workgroups' shares: 16 slices of workgroups per column, then the slices in order
__global__ __launch_bounds__(REDUCE_SLICES* REDUCE_COLS) void reduce_kernel(const float* partials, int n_shares, int gd,
                                                                            float* dgamma, float* dbeta) {
    __shared__ float part[REDUCE_SLICES][REDUCE_COLS];
    const int col = threadIdx.x % REDUCE_COLS, slice = threadIdx.x / REDUCE_COLS;
    const int e = blockIdx.x * REDUCE_COLS + col;
    float s = 0.f;
    if (e < 2 * gd)
        for (int b = slice; b < n_shares; b += REDUCE_SLICES) s += partials[(size_t)b * 2 * gd + e];
    part[slice][col] = s;
    __syncthreads();
    if (slice == 0 && e < 2 * gd) {
        float total = 0.f;
#pragma unroll
        for (int i = 0; i < REDUCE_SLICES; i++) total += part[i][col];
        if (e < gd) dgamma[e] = total;
        else dbeta[e - gd] = total;
    }
}

int grid_for(int64_t n_tokens, int tokens_per_wave) {
    const int64_t per_block = (int64_t)WAVES * tokens_per_wave;
    const int64_t blocks = (n_tokens + per_block - 1) / per_block;
    return (int)(blocks < MAX_BLOCKS ? blocks : MAX_BLOCKS);
}

// Lets `kernel` use the whole 160 KB of LDS as dynamic shared memory.  Asked for once per kernel (the first call is
// not a stream operation, so it is kept out of later calls that a caller may be capturing into a graph).
template <typename KernelT>
hipError_t allow_lds(KernelT kernel) {
    static hipError_t state = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return state;
}

template <typename T, int CPL, bool GATED>
hipError_t launch_fwd_as(const Args& a, hipStream_t s) {
    const size_t lds = (size_t)2 * a.n_groups * a.row * sizeof(float);
    hipError_t e = allow_lds(fwd_kernel<T, CPL, GATED>);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((fwd_kernel<T, CPL, GATED>), dim3(grid_for(a.n, CPL == 1 ? 2 : 1)), dim3(THREADS), lds, s, a);
    return hipGetLastError();
}

template <typename T, int CPL, bool GATED>
hipError_t launch_bwd_as(const Args& a, hipStream_t s) {
    const size_t lds = (size_t)(GATED ? 4 : 3) * a.n_groups * a.row * sizeof(float);
    hipError_t e = allow_lds(bwd_kernel<T, CPL, GATED>);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((bwd_kernel<T, CPL, GATED>), dim3(grid_for(a.n, 1)), dim3(THREADS), lds, s, a);
    return hipGetLastError();
}

template <typename T, bool GATED>
hipError_t dispatch_chunks(bool bwd, const Args& a, hipStream_t s) {
    switch (a.row / CHUNK) {
        case 1: return bwd ? launch_bwd_as<T, 1, GATED>(a, s) : launch_fwd_as<T, 1, GATED>(a, s);
        case 2: return bwd ? launch_bwd_as<T, 2, GATED>(a, s) : launch_fwd_as<T, 2, GATED>(a, s);
        case 3: return bwd ? launch_bwd_as<T, 3, GATED>(a, s) : launch_fwd_as<T, 3, GATED>(a, s);
        default: return bwd ? launch_bwd_as<T, 4, GATED>(a, s) : launch_fwd_as<T, 4, GATED>(a, s);
    }
}

hipError_t dispatch(bool bwd, int dtype, const Args& a, hipStream_t s) {
    const bool gated = a.gate != nullptr;
    if (dtype == MTFM_HTA_BF16)
        return gated ? dispatch_chunks<__bf16, true>(bwd, a, s) : dispatch_chunks<__bf16, false>(bwd, a, s);
    return gated ? dispatch_chunks<float, true>(bwd, a, s) : dispatch_chunks<float, false>(bwd, a, s);
}

int padded_row(int32_t d) { return (d + CHUNK - 1) / CHUNK * CHUNK; }

int check_shape(int64_t n_tokens, int32_t d, int32_t n_groups, int dtype) {
    if (dtype != MTFM_HTA_BF16 && dtype != MTFM_HTA_FP32)
        return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "dtype must be MTFM_HTA_BF16 or MTFM_HTA_FP32, got %d", dtype);
    if (n_tokens < 0) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "negative n_tokens");
    if (d <= 0 || d % 8 != 0)
        return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "d_model must be a positive multiple of 8, got %d", d);
    if (n_groups <= 0) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "n_groups must be positive, got %d", n_groups);
    if (d > CHUNK * MAX_CHUNKS)
        return hta::report_error(MTFM_HTA_ERR_UNSUPPORTED, "d_model %d exceeds %d", d, CHUNK * MAX_CHUNKS);
    if ((int64_t)n_groups * padded_row(d) > MAX_TABLE)
        return hta::report_error(MTFM_HTA_ERR_UNSUPPORTED,
                                 "n_groups (%d) x d_model rounded up to %d (%d) exceeds %d parameter slots in LDS", n_groups,
                                 CHUNK, padded_row(d), MAX_TABLE);
    return MTFM_HTA_OK;
}

bool misaligned(const void* p, unsigned a) { return ((uintptr_t)p & (a - 1)) != 0; }

}  // namespace gln

extern "C" {

int mtfm_gln_fwd(const void* x, const void* gate, const int32_t* group_id, const float* gamma, const float* beta,
                 void* y, float* mean, float* rstd, int64_t n_tokens, int32_t d_model, int32_t n_groups, float eps,
                 int dtype, void* stream) {
    if (int rc = gln::check_shape(n_tokens, d_model, n_groups, dtype)) return rc;
    if (!(eps >= 0.f)) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "eps must be >= 0");
    if (n_tokens == 0) return MTFM_HTA_OK;  // the arrays of an empty call may be null
    if (!x || !group_id || !gamma || !beta || !y) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    if (gln::misaligned(x, 16) || gln::misaligned(gate, 16) || gln::misaligned(y, 16) || gln::misaligned(gamma, 16) ||
        gln::misaligned(beta, 16) || gln::misaligned(group_id, 4) || gln::misaligned(mean, 4) || gln::misaligned(rstd, 4))
        return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "x, gate, y, gamma, beta must be 16-byte aligned");
    gln::Args a = {};
    a.x = x, a.gate = gate, a.group_id = group_id, a.gamma = gamma, a.beta = beta, a.y = y, a.mean = mean, a.rstd = rstd;
    a.n = n_tokens, a.d = d_model, a.n_groups = n_groups, a.row = gln::padded_row(d_model), a.eps = eps;
    hipStream_t s = (hipStream_t)stream;
    hta::timing_begin(MTFM_GLN_KERNEL_FWD, s);
    const hipError_t e = gln::dispatch(false, dtype, a, s);
    hta::timing_end(MTFM_GLN_KERNEL_FWD, s);
    if (e != hipSuccess) return hta::report_error(MTFM_HTA_ERR_LAUNCH, "gln forward launch: %s", hipGetErrorString(e));
    return MTFM_HTA_OK;
}

size_t mtfm_gln_bwd_workspace_bytes(int32_t d_model, int32_t n_groups) {
    if (gln::check_shape(0, d_model, n_groups, MTFM_HTA_BF16) != MTFM_HTA_OK) return 0;
    return (size_t)gln::MAX_BLOCKS * 2 * n_groups * d_model * sizeof(float);
}

int mtfm_gln_bwd(const void* dy, const void* x, const void* gate, const int32_t* group_id, const float* gamma,
                 const float* beta, const float* mean, const float* rstd, void* dx, void* dgate, float* dgamma,
                 float* dbeta, int64_t n_tokens, int32_t d_model, int32_t n_groups, int dtype, void* workspace,
                 size_t workspace_bytes, void* stream) {
    if (int rc = gln::check_shape(n_tokens, d_model, n_groups, dtype)) return rc;
    if (!dgamma || !dbeta) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    // the per-token arrays of an empty call may be null
    if (n_tokens > 0 && (!dy || !x || !group_id || !gamma || !mean || !rstd || !dx))
        return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    if ((gate == nullptr) != (dgate == nullptr))
        return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "gate and dgate must both be given or both be NULL");
    if (gate && !beta) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "beta is required with a gate");
    if (gln::misaligned(dy, 16) || gln::misaligned(x, 16) || gln::misaligned(gate, 16) || gln::misaligned(dx, 16) ||
        gln::misaligned(dgate, 16) || gln::misaligned(gamma, 16) || gln::misaligned(beta, 16) ||
        gln::misaligned(dgamma, 4) || gln::misaligned(dbeta, 4) || gln::misaligned(mean, 4) || gln::misaligned(rstd, 4) ||
        gln::misaligned(group_id, 4))
        return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "dy, x, gate, dx, dgate, gamma, beta must be 16-byte aligned");
    const size_t need = mtfm_gln_bwd_workspace_bytes(d_model, n_groups);
    if (!workspace || workspace_bytes < need)
        return hta::report_error(MTFM_HTA_ERR_WORKSPACE, "this call needs %zu bytes of workspace, got %zu", need,
                                 workspace ? workspace_bytes : (size_t)0);
    if (gln::misaligned(workspace, 256)) return hta::report_error(MTFM_HTA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    gln::Args a = {};
    a.dy = dy, a.x = x, a.gate = gate, a.group_id = group_id, a.gamma = gamma, a.beta = beta, a.mean_in = mean, a.rstd_in = rstd;
    a.dx = dx, a.dgate = dgate, a.partials = (float*)workspace;
    a.n = n_tokens, a.d = d_model, a.n_groups = n_groups, a.row = gln::padded_row(d_model);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    int shares = 0;
    if (n_tokens > 0) {
        // every wave of the grid gets one span when the tokens allow it, several passes of 64 otherwise
        shares = gln::grid_for(n_tokens, 1);
        const int64_t waves = (int64_t)shares * gln::WAVES;
        const int64_t even = (n_tokens + waves - 1) / waves;
        a.span = (int32_t)(even < 64 ? even : 64);
        hta::timing_begin(MTFM_GLN_KERNEL_BWD, s);
        e = gln::dispatch(true, dtype, a, s);
        hta::timing_end(MTFM_GLN_KERNEL_BWD, s);
        if (e != hipSuccess) return hta::report_error(MTFM_HTA_ERR_LAUNCH, "gln backward launch: %s", hipGetErrorString(e));
    }
    const int gd = n_groups * d_model;
    hta::timing_begin(MTFM_GLN_KERNEL_BWD_REDUCE, s);
    hipLaunchKernelGGL(gln::reduce_kernel, dim3((2 * gd + gln::REDUCE_COLS - 1) / gln::REDUCE_COLS),
                       dim3(gln::REDUCE_SLICES * gln::REDUCE_COLS), 0, s, (const float*)workspace, shares, gd, dgamma, dbeta);
    e = hipGetLastError();
    hta::timing_end(MTFM_GLN_KERNEL_BWD_REDUCE, s);
    if (e != hipSuccess) return hta::report_error(MTFM_HTA_ERR_LAUNCH, "gln reduce launch: %s", hipGetErrorString(e));
    return MTFM_HTA_OK;
}

int mtfm_gln_validate_host(const int32_t* group_id, int64_t n_tokens, int32_t n_groups) {
    if (n_tokens < 0 || n_groups <= 0) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "negative n_tokens or n_groups <= 0");
    if (n_tokens > 0 && !group_id) return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "null array");
    for (int64_t i = 0; i < n_tokens; i++)
        if (group_id[i] < 0 || group_id[i] >= n_groups)
            return hta::report_error(MTFM_HTA_ERR_INVALID_ARG, "token %lld: group id %d outside [0, %d)", (long long)i,
                                     group_id[i], n_groups);
    return MTFM_HTA_OK;
}

}  // extern "C"
