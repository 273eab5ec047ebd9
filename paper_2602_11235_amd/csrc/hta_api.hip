// C ABI of libmtfm_hta.so: host-side argument checks and kernel dispatch.  No allocation, no
// host<->device copies, no synchronisation here.
#include "../../include/mtfm_hta.h"
#include "../../include/mtfm_hta_pw.h"
#include "hta_common.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace

namespace hta {
int report_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace hta

namespace {

// head_dim the bf16 kernels run at: 16-wide heads are zero-padded to the 32-wide matrix tiles (copies in the workspace)
inline bool padded_head(int dtype, int32_t d) { return dtype == MTFM_HTA_BF16 && d == hta::BF16_PADDED_FROM; }
inline int32_t kernel_head_dim(int dtype, int32_t d) { return padded_head(dtype, d) ? hta::BF16_PADDED_TO : d; }

// key splits of a forward call, from its host-known bounds (1: none)
int forward_splits(int dtype, int layer, int32_t batch, int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq,
                   int32_t Hkv, int32_t d) {
    if (dtype != MTFM_HTA_BF16) return 1;
    const int64_t keys = (int64_t)max_hist + max_rt;
    const int64_t rows = layer == MTFM_HTA_LAYER_FULL ? keys + max_targets : (int64_t)max_targets;
    return hta::fwd_key_splits(batch, Hq, Hkv, kernel_head_dim(dtype, d), rows, keys);
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
    size_t order_off, delta_off, lse_off, lim_off, opart_off, lsepart_off, total;
    int splits;
    size_t pad_off, pad_q, pad_kv;  // head_dim 16: where the zero-padded copies start, bytes of one q-shaped / kv-shaped copy
};

// Layout of the caller's workspace (bf16 path; the fp32 debug path needs none):
//   work counters (256 bytes) and order [batch] int32, users by decreasing tile count; both rebuilt by every call
//   -delta and -lse/scale, [Hq][total_q] f32 each, the latter followed by one sentinel element   backward only
//   with real-time tokens (both dtypes): lim [total_q] int32, the per-row limits of mask rule 2, rebuilt by every call
//   forward pass split over the keys (`splits` > 1: few requests, decided from the host-known bounds alone):
//   partial outputs [splits][total_q][Hq][d] f32 and their logsumexps [splits][Hq][total_q] f32
//   bf16 head_dim 16: copies of the tensors zero-padded to 32 features, which is what the kernels then see --
//   q, k, v, out (forward); dout, q, k, v, out, dq, dk, dv (backward)
Workspace plan_workspace(int dtype, int is_bwd, int32_t batch, int64_t total_q, int32_t Hq, bool has_rt, int splits = 1,
                         int32_t d = 0, int64_t total_kv = 0, int32_t Hkv = 0) {
    Workspace w{0, 0, 0, 0, 0, 0, 0, 1, 0, 0, 0};
    const bool padded = padded_head(dtype, d);
    d = kernel_head_dim(dtype, d);
    if (has_rt) {
        w.lim_off = 0;
        w.total = align256((size_t)total_q * sizeof(int32_t));
    }
    if (dtype == MTFM_HTA_FP32) return w;
    w.order_off = w.total;
    w.total += hta::schedule_bytes(batch);
    if (is_bwd) {
        w.delta_off = w.total;
        w.total += align256((size_t)total_q * Hq * sizeof(float));
        w.lse_off = w.total;
        w.total += align256(((size_t)total_q * Hq + 1) * sizeof(float));
    } else if (splits > 1) {
        w.splits = splits;
        w.opart_off = w.total;
        w.total += align256((size_t)splits * total_q * Hq * d * sizeof(float));
        w.lsepart_off = w.total;
        w.total += align256((size_t)splits * total_q * Hq * sizeof(float));
    }
    if (padded) {
        w.pad_off = w.total;
        w.pad_q = align256((size_t)total_q * Hq * hta::BF16_PADDED_TO * 2);
        w.pad_kv = align256((size_t)total_kv * Hkv * hta::BF16_PADDED_TO * 2);
        w.total += is_bwd ? 4 * w.pad_q + 4 * w.pad_kv : 2 * w.pad_q + 2 * w.pad_kv;
    }
    return w;
}

int check_workspace(const Workspace& w, const void* workspace, size_t workspace_bytes) {
    if (w.total == 0) return MTFM_HTA_OK;
    if (!workspace || workspace_bytes < w.total)
        return fail(MTFM_HTA_ERR_WORKSPACE, "this call needs %zu bytes of workspace, got %zu", w.total, workspace_bytes);
    if (((uintptr_t)workspace & 255u) != 0) return fail(MTFM_HTA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    return MTFM_HTA_OK;
}

int check_scalars(int layer, int dtype, int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist,
                  int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t d) {
    if (layer != MTFM_HTA_LAYER_FULL && layer != MTFM_HTA_LAYER_TARGET)
        return fail(MTFM_HTA_ERR_INVALID_ARG, "layer must be MTFM_HTA_LAYER_FULL or MTFM_HTA_LAYER_TARGET, got %d", layer);
    if (dtype != MTFM_HTA_BF16 && dtype != MTFM_HTA_FP32)
        return fail(MTFM_HTA_ERR_INVALID_ARG, "dtype must be MTFM_HTA_BF16 or MTFM_HTA_FP32, got %d", dtype);
    if (batch < 0 || total_q < 0 || total_kv < 0 || max_hist < 0 || max_rt < 0 || max_targets < 0)
        return fail(MTFM_HTA_ERR_INVALID_ARG,
                    "negative size (batch %d total_q %lld total_kv %lld max_hist %d max_rt %d max_targets %d)", batch,
                    (long long)total_q, (long long)total_kv, max_hist, max_rt, max_targets);
    if (total_q >= (1ll << 31) || total_kv >= (1ll << 31))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "total_q / total_kv must be below 2^31 (int32 offsets)");
    if (batch > 65535) return fail(MTFM_HTA_ERR_UNSUPPORTED, "batch %d exceeds 65535 users per call", batch);
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0)
        return fail(MTFM_HTA_ERR_INVALID_ARG, "Hq (%d) must be a positive multiple of Hkv (%d)", Hq, Hkv);
    if (Hq > 65535) return fail(MTFM_HTA_ERR_UNSUPPORTED, "Hq %d exceeds 65535", Hq);
    if (d <= 0) return fail(MTFM_HTA_ERR_INVALID_ARG, "head_dim must be positive, got %d", d);
    if (dtype == MTFM_HTA_FP32) {
        if (d > 128) return fail(MTFM_HTA_ERR_UNSUPPORTED, "fp32 path supports head_dim <= 128, got %d", d);
    } else if (!hta::bf16_supported(kernel_head_dim(dtype, d), Hq, Hkv)) {
        return fail(MTFM_HTA_ERR_UNSUPPORTED, "bf16 path supports head_dim in {16, 32, 64, 128}, got %d", d);
    }
    if ((int64_t)max_hist + max_rt + max_targets >= (1ll << 31))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "max_hist + max_rt + max_targets overflows int32");
    return MTFM_HTA_OK;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

}  // namespace

// ---------------------------------------------------------------------------------------------------------------
// mtfm_hta_fwd_static: the forward call for callers that cannot allocate.  What mtfm_hta_fwd keeps in the caller's
// workspace lives in `scratch`, a fixed array in device memory that every GPU the library runs on holds until the
// process ends.  In host code the name `scratch` is only a handle for the runtime, not a device address: the address
// of the array on the current device comes from hipGetSymbolAddress, once per device, and that pointer is what the
// kernels get.
static __device__ __align__(256) unsigned char scratch[MTFM_HTA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch` on each device, resolved on first use

// address of `scratch` on the current device, or null with the error recorded
void* scratch_of_current_device() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        fail(MTFM_HTA_ERR_LAUNCH, "hipGetDevice failed: %s", hipGetErrorString(e));
        return nullptr;
    }
    if (dev < 0 || dev >= MAX_DEVICES) {
        fail(MTFM_HTA_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, MAX_DEVICES - 1);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            fail(MTFM_HTA_ERR_LAUNCH, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

const char* mtfm_hta_last_error(void) { return g_err; }

const char* mtfm_hta_version(void) { return "0.1.0"; }

size_t mtfm_hta_workspace_bytes(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q, int64_t total_kv,
                                int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim) {
    if (check_scalars(layer, dtype, batch, total_q, total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim) != MTFM_HTA_OK)
        return (size_t)-1;
    const int splits = is_bwd ? 1 : forward_splits(dtype, layer, batch, max_hist, 0, max_targets, Hq, Hkv, head_dim);
    return plan_workspace(dtype, is_bwd, batch, total_q, Hq, false, splits, head_dim, total_kv, Hkv).total;
}

size_t mtfm_hta_workspace_bytes_rt(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q, int64_t total_kv,
                                   int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv,
                                   int32_t head_dim) {
    if (check_scalars(layer, dtype, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim) != MTFM_HTA_OK)
        return (size_t)-1;
    const int splits = is_bwd ? 1 : forward_splits(dtype, layer, batch, max_hist, max_rt, max_targets, Hq, Hkv, head_dim);
    return plan_workspace(dtype, is_bwd, batch, total_q, Hq, true, splits, head_dim, total_kv, Hkv).total;
}

static int validate_host_impl(const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                              const int32_t* rt_len, const int32_t* n_targets, const int32_t* timestamps, int32_t batch,
                              int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_rt, int32_t max_targets,
                              int layer) {
    if (batch < 0) return fail(MTFM_HTA_ERR_INVALID_ARG, "negative batch");
    if (layer != MTFM_HTA_LAYER_FULL && layer != MTFM_HTA_LAYER_TARGET)
        return fail(MTFM_HTA_ERR_INVALID_ARG, "bad layer %d", layer);
    if (!q_offsets || !kv_offsets || (batch > 0 && (!hist_len || !n_targets)))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "null array");
    if (rt_len && !timestamps) return fail(MTFM_HTA_ERR_INVALID_ARG, "rt_len without timestamps");
    if (q_offsets[0] != 0 || kv_offsets[0] != 0) return fail(MTFM_HTA_ERR_INVALID_ARG, "offsets must start at 0");
    for (int32_t b = 0; b < batch; b++) {
        const int64_t L = hist_len[b], T = n_targets[b], R = rt_len ? rt_len[b] : 0;
        if (L < 0 || T < 0 || R < 0) return fail(MTFM_HTA_ERR_INVALID_ARG, "user %d: negative length", b);
        if (L > max_hist) return fail(MTFM_HTA_ERR_INVALID_ARG, "user %d: hist_len %lld > max_hist %d", b, (long long)L, max_hist);
        if (R > max_rt) return fail(MTFM_HTA_ERR_INVALID_ARG, "user %d: rt_len %lld > max_rt %d", b, (long long)R, max_rt);
        if (T > max_targets)
            return fail(MTFM_HTA_ERR_INVALID_ARG, "user %d: n_targets %lld > max_targets %d", b, (long long)T, max_targets);
        if ((int64_t)kv_offsets[b + 1] - kv_offsets[b] != L + R + T)
            return fail(MTFM_HTA_ERR_INVALID_ARG, "user %d: kv_offsets span != hist_len + rt_len + n_targets", b);
        const int64_t rows = layer == MTFM_HTA_LAYER_FULL ? L + R + T : T;
        if ((int64_t)q_offsets[b + 1] - q_offsets[b] != rows)
            return fail(MTFM_HTA_ERR_INVALID_ARG, "user %d: q_offsets span %d != %lld query rows", b,
                        q_offsets[b + 1] - q_offsets[b], (long long)rows);
        for (int64_t i = 1; i < R; i++)
            if (timestamps[kv_offsets[b] + L + i] < timestamps[kv_offsets[b] + L + i - 1])
                return fail(MTFM_HTA_ERR_INVALID_ARG, "user %d: real-time tokens are not sorted by timestamp", b);
    }
    if (q_offsets[batch] != total_q) return fail(MTFM_HTA_ERR_INVALID_ARG, "q_offsets[batch] != total_q");
    if (kv_offsets[batch] != total_kv) return fail(MTFM_HTA_ERR_INVALID_ARG, "kv_offsets[batch] != total_kv");
    return MTFM_HTA_OK;
}

int mtfm_hta_validate_host(const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                           const int32_t* n_targets, int32_t batch, int64_t total_q, int64_t total_kv,
                           int32_t max_hist, int32_t max_targets, int layer) {
    return validate_host_impl(q_offsets, kv_offsets, hist_len, nullptr, n_targets, nullptr, batch, total_q, total_kv,
                              max_hist, 0, max_targets, layer);
}

int mtfm_hta_validate_host_rt(const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len,
                              const int32_t* rt_len, const int32_t* n_targets, const int32_t* timestamps, int32_t batch,
                              int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_rt, int32_t max_targets,
                              int layer) {
    if (!rt_len || !timestamps) return fail(MTFM_HTA_ERR_INVALID_ARG, "null array");
    return validate_host_impl(q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps, batch, total_q, total_kv,
                              max_hist, max_rt, max_targets, layer);
}

static int fwd_impl(const void* q, const void* k, const void* v, void* out, float* lse, const int32_t* q_offsets,
                    const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* rt_len, const int32_t* n_targets,
                    const int32_t* timestamps, int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist,
                    int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float softmax_scale,
                    int dtype, int layer, void* workspace, size_t workspace_bytes, void* stream, bool pointwise = false,
                    float norm = 1.f) {
    const bool has_rt = rt_len != nullptr;
    int rc = check_scalars(layer, dtype, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim);
    if (rc != MTFM_HTA_OK) return rc;
    if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "%s must be positive and finite", pointwise ? "scale" : "softmax_scale");
    if (pointwise && (!(norm > 0.f) || !std::isfinite(norm)))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "norm must be positive and finite");
    if (batch == 0 || total_q == 0) return MTFM_HTA_OK;
    if (!q || !k || !v || !out || (!lse && !pointwise) || !q_offsets || !kv_offsets || !hist_len || !n_targets)
        return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "q, k, v, out must be 16-byte aligned");
    if (has_rt && !timestamps) return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    const int splits = forward_splits(dtype, layer, batch, max_hist, max_rt, max_targets, Hq, Hkv, head_dim);
    const Workspace w = plan_workspace(dtype, 0, batch, total_q, Hq, has_rt, splits, head_dim, total_kv, Hkv);
    rc = check_workspace(w, workspace, workspace_bytes);
    if (rc != MTFM_HTA_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    void* const caller_out = out;
    const bool padded = padded_head(dtype, head_dim);
    if (padded) {  // the kernels see copies zero-padded to 32 features; the result is narrowed again at the end
        char* pad = (char*)workspace + w.pad_off;
        void* q32 = pad; void* out32 = pad + w.pad_q; void* k32 = pad + 2 * w.pad_q; void* v32 = pad + 2 * w.pad_q + w.pad_kv;
        e = hta::launch_widen16(q, q32, total_q * Hq, s);
        if (e == hipSuccess) e = hta::launch_widen16(k, k32, total_kv * Hkv, s);
        if (e == hipSuccess) e = hta::launch_widen16(v, v32, total_kv * Hkv, s);
        if (e != hipSuccess) return fail(MTFM_HTA_ERR_LAUNCH, "forward launch failed: %s", hipGetErrorString(e));
        q = q32; k = k32; v = v32; out = out32; head_dim = hta::BF16_PADDED_TO;
    }
    hta::Params p{};
    p.q = q; p.k = k; p.v = v; p.out = out; p.lse = lse;
    p.q_off = q_offsets; p.kv_off = kv_offsets; p.hist_len = hist_len; p.n_targets = n_targets;
    p.batch = batch; p.total_q = total_q; p.total_kv = total_kv; p.max_hist = max_hist; p.max_targets = max_targets;
    p.Hq = Hq; p.Hkv = Hkv; p.d = head_dim; p.scale = softmax_scale; p.layer = layer;
    p.rt_len = rt_len; p.ts = timestamps; p.max_rt = max_rt;
    p.pointwise = pointwise ? 1 : 0; p.norm = norm;
    if (has_rt) {
        p.lim = (int32_t*)((char*)workspace + w.lim_off);
        e = hta::launch_rt_limits(p, s);
    }
    if (e == hipSuccess && dtype == MTFM_HTA_BF16) {
        p.n_splits = w.splits;
        if (w.splits <= 1) {
            void* region = (char*)workspace + w.order_off;
            e = hta::launch_schedule(p, region, s);
            p.order = hta::schedule_order(region);
            p.queue = hta::schedule_queue(region, 0);  // the launchers add the kernel kind
        } else {
            // a few users that do not fill the chip anyway: no long-first order (p.order stays null = as given),
            // and one kernel less on the critical path of the call
            p.o_part = (float*)((char*)workspace + w.opart_off);
            p.lse_part = (float*)((char*)workspace + w.lsepart_off);
        }
    }
    if (e == hipSuccess) e = dtype == MTFM_HTA_FP32 ? hta::launch_fwd_fp32(p, s) : hta::launch_fwd_bf16(p, s);
    if (e == hipSuccess && padded) e = hta::launch_narrow16(out, caller_out, total_q * Hq, s);
    if (e != hipSuccess) return fail(MTFM_HTA_ERR_LAUNCH, "forward launch failed: %s", hipGetErrorString(e));
    return MTFM_HTA_OK;
}

int mtfm_hta_fwd(const void* q, const void* k, const void* v, void* out, float* lse, const int32_t* q_offsets,
                 const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* n_targets, int32_t batch,
                 int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv,
                 int32_t head_dim, float softmax_scale, int dtype, int layer, void* workspace, size_t workspace_bytes,
                 void* stream) {
    return fwd_impl(q, k, v, out, lse, q_offsets, kv_offsets, hist_len, nullptr, n_targets, nullptr, batch, total_q,
                    total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer, workspace,
                    workspace_bytes, stream);
}

int mtfm_hta_fwd_static(const void* q, const void* k, const void* v, void* out, float* lse, const int32_t* q_offsets,
                        const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* n_targets, int32_t batch,
                        int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_targets, int32_t Hq,
                        int32_t Hkv, int32_t head_dim, float softmax_scale, int dtype, int layer, void* stream) {
    int rc = check_scalars(layer, dtype, batch, total_q, total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim);
    if (rc != MTFM_HTA_OK) return rc;
    const int splits = forward_splits(dtype, layer, batch, max_hist, 0, max_targets, Hq, Hkv, head_dim);
    const size_t need = plan_workspace(dtype, 0, batch, total_q, Hq, false, splits, head_dim, total_kv, Hkv).total;
    if (need > (size_t)MTFM_HTA_STATIC_SCRATCH_BYTES)
        return fail(MTFM_HTA_ERR_WORKSPACE,
                    "mtfm_hta_fwd_static: this call needs %zu bytes of scratch memory, the built-in buffer holds %zu; "
                    "use mtfm_hta_fwd with a workspace of the caller's", need, (size_t)MTFM_HTA_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if (need > 0 && batch > 0 && total_q > 0) {
        ws = scratch_of_current_device();
        if (!ws) return MTFM_HTA_ERR_LAUNCH;
    }
    // Everything the kernels expect to find zeroed in the scratch memory (the work counters) is cleared by the
    // schedule kernel at the start of the call; the rest is written before it is read.
    return fwd_impl(q, k, v, out, lse, q_offsets, kv_offsets, hist_len, nullptr, n_targets, nullptr, batch, total_q,
                    total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer, ws,
                    ws ? (size_t)MTFM_HTA_STATIC_SCRATCH_BYTES : 0, stream);
}

int mtfm_hta_fwd_rt(const void* q, const void* k, const void* v, void* out, float* lse, const int32_t* q_offsets,
                    const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* rt_len, const int32_t* n_targets,
                    const int32_t* timestamps, int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist,
                    int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float softmax_scale,
                    int dtype, int layer, void* workspace, size_t workspace_bytes, void* stream) {
    if (batch > 0 && total_q > 0 && (!rt_len || !timestamps)) return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    return fwd_impl(q, k, v, out, lse, q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps, batch, total_q,
                    total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer, workspace,
                    workspace_bytes, stream);
}

static int bwd_impl(const void* dout, const void* q, const void* k, const void* v, const void* out, const float* lse,
                    void* dq, void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets,
                    const int32_t* hist_len, const int32_t* rt_len, const int32_t* n_targets, const int32_t* timestamps,
                    int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_rt,
                    int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float softmax_scale, int dtype,
                    int layer, void* workspace, size_t workspace_bytes, void* stream, bool pointwise = false,
                    float norm = 1.f) {
    const bool has_rt = rt_len != nullptr;
    int rc = check_scalars(layer, dtype, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim);
    if (rc != MTFM_HTA_OK) return rc;
    if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "%s must be positive and finite", pointwise ? "scale" : "softmax_scale");
    if (pointwise && (!(norm > 0.f) || !std::isfinite(norm)))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "norm must be positive and finite");
    if (batch == 0 || total_kv == 0) return MTFM_HTA_OK;
    // a target layer whose users have no candidate at all has no query row (total_q == 0): the row-shaped tensors are
    // empty then and may be null; dk = dv = 0 is still written
    const bool no_rows = total_q == 0;
    if ((!no_rows && (!dout || !q || (!pointwise && (!out || !lse)) || !dq)) || !k || !v || !dk || !dv || !q_offsets ||
        !kv_offsets || !hist_len || !n_targets)
        return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    if (misaligned(dout) || misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(dq) ||
        misaligned(dk) || misaligned(dv))
        return fail(MTFM_HTA_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (has_rt && !timestamps) return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    const Workspace w = plan_workspace(dtype, 1, batch, total_q, Hq, has_rt, 1, head_dim, total_kv, Hkv);
    rc = check_workspace(w, workspace, workspace_bytes);
    if (rc != MTFM_HTA_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    void* const caller_dq = dq; void* const caller_dk = dk; void* const caller_dv = dv;
    const bool padded = padded_head(dtype, head_dim);
    if (padded) {  // as in the forward call: the kernels see zero-padded copies, the gradients are narrowed at the end
        char* pad = (char*)workspace + w.pad_off;
        void* dout32 = pad; void* q32 = pad + w.pad_q; void* out32 = pad + 2 * w.pad_q; void* dq32 = pad + 3 * w.pad_q;
        char* kv = pad + 4 * w.pad_q;
        void* k32 = kv; void* v32 = kv + w.pad_kv; void* dk32 = kv + 2 * w.pad_kv; void* dv32 = kv + 3 * w.pad_kv;
        e = hta::launch_widen16(dout, dout32, total_q * Hq, s);
        if (e == hipSuccess) e = hta::launch_widen16(q, q32, total_q * Hq, s);
        if (e == hipSuccess && out) e = hta::launch_widen16(out, out32, total_q * Hq, s);
        if (e == hipSuccess) e = hta::launch_widen16(k, k32, total_kv * Hkv, s);
        if (e == hipSuccess) e = hta::launch_widen16(v, v32, total_kv * Hkv, s);
        if (e != hipSuccess) return fail(MTFM_HTA_ERR_LAUNCH, "backward launch failed: %s", hipGetErrorString(e));
        dout = dout32; q = q32; k = k32; v = v32; if (out) out = out32;
        dq = dq32; dk = dk32; dv = dv32; head_dim = hta::BF16_PADDED_TO;
    }
    hta::Params p{};
    p.dout = dout; p.q = q; p.k = k; p.v = v; p.out = const_cast<void*>(out); p.lse = const_cast<float*>(lse);
    p.dq = dq; p.dk = dk; p.dv = dv;
    p.q_off = q_offsets; p.kv_off = kv_offsets; p.hist_len = hist_len; p.n_targets = n_targets;
    p.batch = batch; p.total_q = total_q; p.total_kv = total_kv; p.max_hist = max_hist; p.max_targets = max_targets;
    p.Hq = Hq; p.Hkv = Hkv; p.d = head_dim; p.scale = softmax_scale; p.layer = layer;
    p.rt_len = rt_len; p.ts = timestamps; p.max_rt = max_rt;
    p.pointwise = pointwise ? 1 : 0; p.norm = norm;
    if (dtype == MTFM_HTA_BF16) {
        char* base = (char*)workspace;
        p.neg_delta = (float*)(base + w.delta_off);
        p.neg_lse_s = (float*)(base + w.lse_off);
    }
    if (has_rt) {
        p.lim = (int32_t*)((char*)workspace + w.lim_off);
        e = hta::launch_rt_limits(p, s);
    }
    if (e == hipSuccess && dtype == MTFM_HTA_BF16) {
        void* region = (char*)workspace + w.order_off;
        e = hta::launch_schedule(p, region, s);
        p.order = hta::schedule_order(region);
        p.queue = hta::schedule_queue(region, 0);  // the launchers add the kernel kind
    }
    if (e == hipSuccess) e = dtype == MTFM_HTA_FP32 ? hta::launch_bwd_fp32(p, s) : hta::launch_bwd_bf16(p, s);
    if (e == hipSuccess && padded) {
        e = hta::launch_narrow16(dq, caller_dq, total_q * Hq, s);
        if (e == hipSuccess) e = hta::launch_narrow16(dk, caller_dk, total_kv * Hkv, s);
        if (e == hipSuccess) e = hta::launch_narrow16(dv, caller_dv, total_kv * Hkv, s);
    }
    if (e != hipSuccess) return fail(MTFM_HTA_ERR_LAUNCH, "backward launch failed: %s", hipGetErrorString(e));
    return MTFM_HTA_OK;
}

int mtfm_hta_bwd(const void* dout, const void* q, const void* k, const void* v, const void* out, const float* lse,
                 void* dq, void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets,
                 const int32_t* hist_len, const int32_t* n_targets, int32_t batch, int64_t total_q, int64_t total_kv,
                 int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float softmax_scale,
                 int dtype, int layer, void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(dout, q, k, v, out, lse, dq, dk, dv, q_offsets, kv_offsets, hist_len, nullptr, n_targets, nullptr,
                    batch, total_q, total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer,
                    workspace, workspace_bytes, stream);
}

int mtfm_hta_bwd_rt(const void* dout, const void* q, const void* k, const void* v, const void* out, const float* lse,
                    void* dq, void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets,
                    const int32_t* hist_len, const int32_t* rt_len, const int32_t* n_targets, const int32_t* timestamps,
                    int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_rt,
                    int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float softmax_scale, int dtype,
                    int layer, void* workspace, size_t workspace_bytes, void* stream) {
    if (batch > 0 && total_kv > 0 && (!rt_len || !timestamps)) return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    return bwd_impl(dout, q, k, v, out, lse, dq, dk, dv, q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps,
                    batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim, softmax_scale, dtype, layer,
                    workspace, workspace_bytes, stream);
}

size_t mtfm_hta_pw_workspace_bytes(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q, int64_t total_kv,
                                   int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim) {
    if (check_scalars(layer, dtype, batch, total_q, total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim) != MTFM_HTA_OK)
        return (size_t)-1;
    const int splits = is_bwd ? 1 : forward_splits(dtype, layer, batch, max_hist, 0, max_targets, Hq, Hkv, head_dim);
    return plan_workspace(dtype, is_bwd, batch, total_q, Hq, false, splits, head_dim, total_kv, Hkv).total;
}

int mtfm_hta_pw_fwd(const void* q, const void* k, const void* v, void* out, const int32_t* q_offsets,
                    const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* n_targets, int32_t batch,
                    int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_targets, int32_t Hq, int32_t Hkv,
                    int32_t head_dim, float scale, float norm, int dtype, int layer, void* workspace,
                    size_t workspace_bytes, void* stream) {
    return fwd_impl(q, k, v, out, nullptr, q_offsets, kv_offsets, hist_len, nullptr, n_targets, nullptr, batch, total_q,
                    total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim, scale, dtype, layer, workspace, workspace_bytes,
                    stream, true, norm);
}

int mtfm_hta_pw_bwd(const void* dout, const void* q, const void* k, const void* v, void* dq, void* dk, void* dv,
                    const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* n_targets,
                    int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist, int32_t max_targets, int32_t Hq,
                    int32_t Hkv, int32_t head_dim, float scale, float norm, int dtype, int layer, void* workspace,
                    size_t workspace_bytes, void* stream) {
    return bwd_impl(dout, q, k, v, nullptr, nullptr, dq, dk, dv, q_offsets, kv_offsets, hist_len, nullptr, n_targets,
                    nullptr, batch, total_q, total_kv, max_hist, 0, max_targets, Hq, Hkv, head_dim, scale, dtype, layer,
                    workspace, workspace_bytes, stream, true, norm);
}

size_t mtfm_hta_pw_workspace_bytes_rt(int layer, int dtype, int is_bwd, int32_t batch, int64_t total_q, int64_t total_kv,
                                      int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv,
                                      int32_t head_dim) {
    if (check_scalars(layer, dtype, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim) != MTFM_HTA_OK)
        return (size_t)-1;
    const int splits = is_bwd ? 1 : forward_splits(dtype, layer, batch, max_hist, max_rt, max_targets, Hq, Hkv, head_dim);
    return plan_workspace(dtype, is_bwd, batch, total_q, Hq, true, splits, head_dim, total_kv, Hkv).total;
}

int mtfm_hta_pw_fwd_rt(const void* q, const void* k, const void* v, void* out, const int32_t* q_offsets,
                       const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* rt_len, const int32_t* n_targets,
                       const int32_t* timestamps, int32_t batch, int64_t total_q, int64_t total_kv, int32_t max_hist,
                       int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim, float scale,
                       float norm, int dtype, int layer, void* workspace, size_t workspace_bytes, void* stream) {
    if (batch > 0 && total_q > 0 && (!rt_len || !timestamps)) return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    return fwd_impl(q, k, v, out, nullptr, q_offsets, kv_offsets, hist_len, rt_len, n_targets, timestamps, batch, total_q,
                    total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim, scale, dtype, layer, workspace,
                    workspace_bytes, stream, true, norm);
}

int mtfm_hta_pw_bwd_rt(const void* dout, const void* q, const void* k, const void* v, void* dq, void* dk, void* dv,
                       const int32_t* q_offsets, const int32_t* kv_offsets, const int32_t* hist_len, const int32_t* rt_len,
                       const int32_t* n_targets, const int32_t* timestamps, int32_t batch, int64_t total_q, int64_t total_kv,
                       int32_t max_hist, int32_t max_rt, int32_t max_targets, int32_t Hq, int32_t Hkv, int32_t head_dim,
                       float scale, float norm, int dtype, int layer, void* workspace, size_t workspace_bytes,
                       void* stream) {
    if (batch > 0 && total_kv > 0 && (!rt_len || !timestamps)) return fail(MTFM_HTA_ERR_INVALID_ARG, "null pointer argument");
    return bwd_impl(dout, q, k, v, nullptr, nullptr, dq, dk, dv, q_offsets, kv_offsets, hist_len, rt_len, n_targets,
                    timestamps, batch, total_q, total_kv, max_hist, max_rt, max_targets, Hq, Hkv, head_dim, scale, dtype,
                    layer, workspace, workspace_bytes, stream, true, norm);
}

}  // extern "C"
