// float32 debug path of Hybrid Target Attention: plain FMA arithmetic, one wavefront per
// (query row, query head).  It exists to check the jagged indexing, the hybrid mask and the
// C ABI independently of the MFMA kernels; it is not tuned.
//
// Mask rules (Section 3.2.2): the keys a query token `tok` may attend to are the L_b history tokens
// (rule 1), the real-time tokens strictly earlier than it (rule 2; a prefix of the time-sorted real-time
// segment that follows the history), plus itself when it is a real-time or target token (tok >= L_b).  So
// the visible keys of a row are the list [0, lead) followed by at most one more entry, `tok` itself, with
// lead = L_b without real-time tokens and the precomputed per-row limit otherwise.
#include "../../include/mtfm_hta.h"
#include "../../include/mtfm_hta_timing.h"
#include "hta_common.h"

namespace hta {
namespace {

constexpr int WAVE = 64;

__device__ inline float wave_max(float x) {
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ inline float wave_sum(float x) {
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

struct RowInfo {
    bool valid;
    int64_t q_row;     // row in the packed q/out tensors
    int64_t kv_base;   // first K/V row of the user
    int32_t L;         // leading K/V rows of the user that the row sees
    int32_t tok;       // token index of the query inside the user's sample
    int32_t n_vis;     // number of visible keys
};

__device__ inline RowInfo locate_row(const Params& p, int b, int64_t row) {
    RowInfo r;
    const int32_t L = p.hist_len[b], T = p.n_targets[b], R = p.rt_len ? p.rt_len[b] : 0;
    const int64_t n_rows = p.layer == 0 ? (int64_t)L + R + T : T;
    r.valid = row < n_rows;
    r.tok = p.layer == 0 ? (int32_t)row : L + R + (int32_t)row;
    r.q_row = (int64_t)p.q_off[b] + row;
    r.kv_base = p.kv_off[b];
    r.L = (p.lim && r.valid) ? p.lim[r.q_row] : L;
    r.n_vis = r.L + (r.tok >= L ? 1 : 0);
    return r;
}

// grid: x = query row within the user (up to the host-known bound), y = query head, z = user
template <int DMAX>
__global__ __launch_bounds__(WAVE) void fwd_fp32_kernel(Params p) {
    const int b = blockIdx.z, h = blockIdx.y, lane = threadIdx.x;
    const RowInfo ri = locate_row(p, b, blockIdx.x);
    if (!ri.valid) return;
    const int d = p.d, g = h / (p.Hq / p.Hkv);
    const float* q = (const float*)p.q + (ri.q_row * p.Hq + h) * d;
    const float* kb = (const float*)p.k + (ri.kv_base * p.Hkv + g) * d;
    const float* vb = (const float*)p.v + (ri.kv_base * p.Hkv + g) * d;
    const int64_t kv_stride = (int64_t)p.Hkv * d;
    float qr[DMAX];
#pragma unroll
    for (int c = 0; c < DMAX; c++) qr[c] = c < d ? q[c] : 0.f;

    if (p.pointwise) {  // out = norm * sum over the visible keys of silu(scale <q, k>) v
        float acc[DMAX];
#pragma unroll
        for (int c = 0; c < DMAX; c++) acc[c] = 0.f;
        for (int idx = lane; idx < ri.n_vis; idx += WAVE) {
            const int key = idx < ri.L ? idx : ri.tok;
            const float* kj = kb + key * kv_stride;
            const float* vj = vb + key * kv_stride;
            float dot = 0.f;
#pragma unroll
            for (int c = 0; c < DMAX; c++)
                if (c < d) dot = fmaf(qr[c], kj[c], dot);
            const float x = p.scale * dot;
            const float w = p.norm * x / (1.f + expf(-x));
#pragma unroll
            for (int c = 0; c < DMAX; c++)
                if (c < d) acc[c] = fmaf(w, vj[c], acc[c]);
        }
        float* o = (float*)p.out + (ri.q_row * p.Hq + h) * d;
#pragma unroll
        for (int c = 0; c < DMAX; c++) {
            if (c < d) {
                const float s = wave_sum(acc[c]);
                if (lane == 0) o[c] = s;
            }
        }
        return;
    }
    // pass 1: row maximum of the scaled logits
    float m = -INFINITY;
    for (int idx = lane; idx < ri.n_vis; idx += WAVE) {
        const int key = idx < ri.L ? idx : ri.tok;
        const float* kj = kb + key * kv_stride;
        float dot = 0.f;
#pragma unroll
        for (int c = 0; c < DMAX; c++)
            if (c < d) dot = fmaf(qr[c], kj[c], dot);
        m = fmaxf(m, p.scale * dot);
    }
    m = wave_max(m);
    // pass 2: weights and weighted sum of value rows
    float l = 0.f, acc[DMAX];
#pragma unroll
    for (int c = 0; c < DMAX; c++) acc[c] = 0.f;
    for (int idx = lane; idx < ri.n_vis; idx += WAVE) {
        const int key = idx < ri.L ? idx : ri.tok;
        const float* kj = kb + key * kv_stride;
        const float* vj = vb + key * kv_stride;
        float dot = 0.f;
#pragma unroll
        for (int c = 0; c < DMAX; c++)
            if (c < d) dot = fmaf(qr[c], kj[c], dot);
        const float w = expf(p.scale * dot - m);
        l += w;
#pragma unroll
        for (int c = 0; c < DMAX; c++)
            if (c < d) acc[c] = fmaf(w, vj[c], acc[c]);
    }
    l = wave_sum(l);
    float* o = (float*)p.out + (ri.q_row * p.Hq + h) * d;
#pragma unroll
    for (int c = 0; c < DMAX; c++) {
        if (c < d) {
            const float s = wave_sum(acc[c]);
            if (lane == 0) o[c] = s / l;
        }
    }
    if (lane == 0) p.lse[(int64_t)h * p.total_q + ri.q_row] = m + logf(l);
}

// Same grid.  dk/dv (float32) must be zero on entry: every visible (row, key) pair adds its term
// with an atomic.
template <int DMAX>
__global__ __launch_bounds__(WAVE) void bwd_fp32_kernel(Params p) {
    const int b = blockIdx.z, h = blockIdx.y, lane = threadIdx.x;
    const RowInfo ri = locate_row(p, b, blockIdx.x);
    if (!ri.valid) return;
    const int d = p.d, g = h / (p.Hq / p.Hkv);
    const int64_t qo = (ri.q_row * p.Hq + h) * d;
    const float* q = (const float*)p.q + qo;
    const float* dout = (const float*)p.dout + qo;
    const float* out = p.pointwise ? nullptr : (const float*)p.out + qo;
    const int64_t kv_stride = (int64_t)p.Hkv * d;
    const int64_t kvo = (ri.kv_base * p.Hkv + g) * d;
    const float* kb = (const float*)p.k + kvo;
    const float* vb = (const float*)p.v + kvo;
    float* dkb = (float*)p.dk + kvo;
    float* dvb = (float*)p.dv + kvo;
    float qr[DMAX], dor[DMAX], dqa[DMAX];
    float delta = 0.f;
#pragma unroll
    for (int c = 0; c < DMAX; c++) {
        qr[c] = c < d ? q[c] : 0.f;
        dor[c] = c < d ? dout[c] : 0.f;
        dqa[c] = 0.f;
        if (c < d && out) delta = fmaf(dor[c], out[c], delta);
    }
    const float lse = p.pointwise ? 0.f : p.lse[(int64_t)h * p.total_q + ri.q_row];
    for (int idx = lane; idx < ri.n_vis; idx += WAVE) {
        const int key = idx < ri.L ? idx : ri.tok;
        const float* kj = kb + key * kv_stride;
        const float* vj = vb + key * kv_stride;
        float dot = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < DMAX; c++) {
            if (c < d) {
                dot = fmaf(qr[c], kj[c], dot);
                dp = fmaf(dor[c], vj[c], dp);
            }
        }
        float w, ds;
        if (p.pointwise) {  // w = norm silu(x), ds = norm dp silu'(x)
            const float x = p.scale * dot;
            const float sg = 1.f / (1.f + expf(-x));
            w = p.norm * x * sg;
            ds = p.norm * dp * sg * (1.f + x * (1.f - sg));
        } else {
            w = expf(p.scale * dot - lse);
            ds = w * (dp - delta);
        }
        const float sds = p.scale * ds;
#pragma unroll
        for (int c = 0; c < DMAX; c++) {
            if (c < d) {
                dqa[c] = fmaf(ds, kj[c], dqa[c]);
                atomicAdd(dkb + key * kv_stride + c, sds * qr[c]);
                atomicAdd(dvb + key * kv_stride + c, w * dor[c]);
            }
        }
    }
    float* dq = (float*)p.dq + qo;
#pragma unroll
    for (int c = 0; c < DMAX; c++) {
        if (c < d) {
            const float s = wave_sum(dqa[c]);
            if (lane == 0) dq[c] = p.scale * s;
        }
    }
}

__global__ void zero_words_kernel(uint32_t* ptr, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) ptr[i] = 0u;
}

template <int DMAX>
hipError_t launch_pair(const Params& p, hipStream_t s, bool bwd) {
    const int64_t rows = max_query_rows(p);
    if (rows <= 0 || p.batch <= 0) return hipSuccess;
    dim3 grid((unsigned)rows, (unsigned)p.Hq, (unsigned)p.batch);
    if (bwd)
        hipLaunchKernelGGL(bwd_fp32_kernel<DMAX>, grid, dim3(WAVE), 0, s, p);
    else
        hipLaunchKernelGGL(fwd_fp32_kernel<DMAX>, grid, dim3(WAVE), 0, s, p);
    return hipGetLastError();
}

hipError_t dispatch(const Params& p, hipStream_t s, bool bwd) {
    if (p.d <= 16) return launch_pair<16>(p, s, bwd);
    if (p.d <= 32) return launch_pair<32>(p, s, bwd);
    if (p.d <= 64) return launch_pair<64>(p, s, bwd);
    return launch_pair<128>(p, s, bwd);
}

}  // namespace

hipError_t launch_zero_words(void* ptr, size_t n_words, hipStream_t s) {
    if (n_words == 0) return hipSuccess;
    size_t blocks = (n_words + 256 * 8 - 1) / (256 * 8);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint32_t*)ptr, n_words);
    return hipGetLastError();
}

hipError_t launch_fwd_fp32(const Params& p, hipStream_t s) {
    timing_begin(MTFM_HTA_KERNEL_FWD, s);
    const hipError_t e = dispatch(p, s, false);
    timing_end(MTFM_HTA_KERNEL_FWD, s);
    return e;
}

hipError_t launch_bwd_fp32(const Params& p, hipStream_t s) {
    hipError_t e = launch_zero_words(p.dk, (size_t)p.total_kv * p.Hkv * p.d, s);
    if (e != hipSuccess) return e;
    e = launch_zero_words(p.dv, (size_t)p.total_kv * p.Hkv * p.d, s);
    if (e != hipSuccess) return e;
    timing_begin(MTFM_HTA_KERNEL_BWD_DQ, s);
    e = dispatch(p, s, true);
    timing_end(MTFM_HTA_KERNEL_BWD_DQ, s);
    return e;
}

}  // namespace hta
