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
    float* neg_delta;     // [Hq][total_q]   -<dout_i, out_i>
    float* neg_lse_s;     // [Hq][total_q]   -lse_i / scale: what the S accumulators of the dK/dV pass start from
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
// Placement of workgroups.  Work is a list of groups (user slot, y) -- y = kv head (x head chunk) -- each with up
// to `tpg` tiles that share operands (the K/V of the group, or its Q/dO).  The chip has 8 XCDs, each with its own
// L2, and hands consecutive workgroup ids to them round-robin; so id -> (xcd = id % 8, slot = id / 8), a group lives
// on one XCD (its tiles are consecutive slots there, so they also run close in time), and groups are dealt to the
// XCDs round-robin in schedule order, which keeps the long-first order inside every XCD.  Only locality depends
// on the round-robin assumption, never correctness.
constexpr int N_XCD = 8;
struct WorkItem {
    int user_slot, y, tile;
    bool valid;
};
__device__ inline WorkItem decode_work(unsigned id, int n_groups, int ny, int tpg) {
    const int xcd = id % N_XCD, slot = id / N_XCD;
    const int gl = slot / tpg;
    const int group = gl * N_XCD + xcd;
    WorkItem w;
    w.valid = group < n_groups;
    w.tile = slot - gl * tpg;
    w.user_slot = group / ny;
    w.y = group - w.user_slot * ny;
    return w;
}
inline int64_t work_grid(int64_t n_groups, int64_t tpg) { return ((n_groups + N_XCD - 1) / N_XCD) * N_XCD * tpg; }
// fill `n` 32-bit words with zero (a kernel, so that a caller may capture the call in a HIP graph)
hipError_t launch_zero_words(void* ptr, size_t n_words, hipStream_t s);

}  // namespace hta
