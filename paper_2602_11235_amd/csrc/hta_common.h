// Internal declarations shared by the translation units of libmtfm_hta.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hta {

// Everything one call needs, passed to the kernels by value.
struct Params {
    const void* q;
    const void* k;
    const void* v;
    void* out;            // fwd: output; bwd: the saved forward output (read only)
    float* lse;           // [Hq][total_q]
    const void* dout;     // bwd only
    void* dq;
    void* dk;
    void* dv;
    const int32_t* q_off;   // [B+1]
    const int32_t* kv_off;  // [B+1]
    const int32_t* hist_len;
    const int32_t* n_targets;
    int32_t batch;
    int64_t total_q;
    int64_t total_kv;
    int32_t max_hist;
    int32_t max_targets;
    int32_t Hq;
    int32_t Hkv;
    int32_t d;
    float scale;
    int32_t layer;        // 0 full (queries = all tokens), 1 target (queries = target tokens)
    // carved out of the caller's workspace (bwd)
    float* delta;         // [Hq][total_q]   <dout_i, out_i>
    const int32_t* order; // [batch] users by decreasing tile count (bf16 path), or null = identity
};

// number of query rows a user can have at most, from the host-known bounds
inline int64_t max_query_rows(const Params& p) {
    return p.layer == 0 ? (int64_t)p.max_hist + p.max_targets : (int64_t)p.max_targets;
}

hipError_t launch_fwd_fp32(const Params& p, hipStream_t s);
hipError_t launch_bwd_fp32(const Params& p, hipStream_t s);
hipError_t launch_fwd_bf16(const Params& p, hipStream_t s);
hipError_t launch_bwd_bf16(const Params& p, hipStream_t s);
bool bf16_supported(int32_t d, int32_t Hq, int32_t Hkv);
// event hooks around each kernel (no-ops unless timing was enabled through the C ABI); `kind` is one of the
// MTFM_HTA_KERNEL_* values
void timing_begin(int kind, hipStream_t s);
void timing_end(int kind, hipStream_t s);
// user order of the launch (blockIdx.z -> user): long histories first
size_t schedule_bytes(int32_t batch);
hipError_t launch_schedule(const Params& p, int32_t* order, hipStream_t s);
__device__ inline int scheduled_user(const Params& p, int slot) { return p.order ? p.order[slot] : slot; }
// fill `n` 32-bit words with zero (a kernel, so that a caller may capture the call in a HIP graph)
hipError_t launch_zero_words(void* ptr, size_t n_words, hipStream_t s);

}  // namespace hta
