// Internal declarations shared by the translation units of libmtfm_hta.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

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
    int32_t* queue;       // [N_XCD] work counters of the kernel being launched (bf16 path), zero when it starts
    // real-time tokens (mask rule 2); all null / 0 for samples of history + target tokens only
    const int32_t* rt_len;  // [B] real-time tokens of each user, between its history and its target tokens
    const int32_t* ts;      // [total_kv] one timestamp per K/V row
    int32_t max_rt;
    // the pointwise reading of phi2: weights norm * silu(scale s) instead of a row softmax (no lse, no delta)
    int32_t pointwise;
    float norm;
    // forward pass split over the keys (few requests: inference); n_splits <= 1 = not split
    int32_t n_splits;
    float* o_part;          // [n_splits][total_q][Hq][d] partial outputs, each normalised by its own sum
    float* lse_part;        // [n_splits][Hq][total_q]    logsumexp of each split's keys (-inf: none)
    int32_t* lim;           // [total_q] carved out of the workspace: number of leading K/V rows of the user (history, then
                            // the real-time tokens strictly earlier than the query) that the query row sees
};

// number of query rows a user can have at most, from the host-known bounds
__host__ __device__ inline int64_t max_query_rows(const Params& p) {
    return p.layer == 0 ? (int64_t)p.max_hist + p.max_rt + p.max_targets : (int64_t)p.max_targets;
}
// number of keys a user's tile loops can reach at most: history, then real-time tokens
__host__ __device__ inline int64_t max_lead_keys(const Params& p) { return (int64_t)p.max_hist + p.max_rt; }
// per-row limits of mask rule 2 (a launch of its own at the start of a call with real-time tokens)
hipError_t launch_rt_limits(const Params& p, hipStream_t s);

hipError_t launch_fwd_fp32(const Params& p, hipStream_t s);
hipError_t launch_bwd_fp32(const Params& p, hipStream_t s);
hipError_t launch_fwd_bf16(const Params& p, hipStream_t s);
hipError_t launch_bwd_bf16(const Params& p, hipStream_t s);
// the two launches of launch_bwd_bf16 that live in translation units of their own (other compiler options)
hipError_t launch_bwd_dq_bf16(const Params& p, hipStream_t s);       // dQ and the self-key blocks, every head_dim
hipError_t launch_bwd_dkdv128_bf16(const Params& p, hipStream_t s);  // dK/dV at head_dim 128, softmax weights, no real-time tokens
bool bf16_supported(int32_t d, int32_t Hq, int32_t Hkv);
// bf16 rows of 16 features <-> rows of 32 with a zero upper half ([n_rows][16] and [n_rows][32], 16-byte aligned): how
// head_dim 16 rides the 32-wide matrix tiles
constexpr int32_t BF16_PADDED_FROM = 16, BF16_PADDED_TO = 32;
hipError_t launch_widen16(const void* src, void* dst, int64_t n_rows, hipStream_t s);
hipError_t launch_narrow16(const void* src, void* dst, int64_t n_rows, hipStream_t s);
// number of key splits the bf16 forward pass uses for these host-known bounds (1 = none); decides the workspace too
int fwd_key_splits(int32_t batch, int32_t Hq, int32_t Hkv, int32_t d, int64_t max_rows, int64_t max_keys);
// stores the calling thread's error message (what mtfm_hta_last_error() returns) and hands `code` back
int report_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
// event hooks around each kernel (no-ops unless timing was enabled through the C ABI); `kind` is one of the
// MTFM_HTA_KERNEL_* values
void timing_begin(int kind, hipStream_t s);
void timing_end(int kind, hipStream_t s);
// The schedule region at the head of the workspace: work counters (one per kernel kind and XCD, 256 bytes in all),
// then the user order of the launch, long histories first.  launch_schedule() zeroes the former and builds the latter.
constexpr int N_XCD = 8;
constexpr int QUEUE_DKDV = 0;  // kernel kinds that take their work from counters
constexpr int QUEUE_WORDS = 64;
size_t schedule_bytes(int32_t batch);
hipError_t launch_schedule(const Params& p, void* region, hipStream_t s);
inline int32_t* schedule_order(void* region) { return (int32_t*)region + QUEUE_WORDS; }
inline int32_t* schedule_queue(void* region, int kind) { return (int32_t*)region + kind * N_XCD; }
__device__ inline int scheduled_user(const Params& p, int slot) { return p.order ? p.order[slot] : slot; }
// Placement of workgroups.  Work is a list of groups (user slot, y) -- y = kv head (x head chunk) -- each with up
// to `tpg` tiles that share operands (the K/V of the group, or its Q/dO).  The chip has 8 XCDs, each with its own
// L2, and hands consecutive workgroup ids to them round-robin; so id -> (xcd = id % 8, slot = id / 8), a group lives
// on one XCD (its tiles are consecutive slots there, so they also run close in time), and groups are dealt to the
// XCDs round-robin in schedule order, which keeps the long-first order inside every XCD.  Only locality depends
// on the round-robin assumption, never correctness.
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

// Work distribution for kernels with long work items (the dK/dV pass: tens of microseconds per item).  The hardware
// hands the workgroups of a grid to the shader engines in a fixed rotation, whatever each has left to do, so with items
// of unequal length (jagged users) whole compute units run dry while others queue up: a fifth of the chip on the
// paper's length mix.  Such a kernel launches only as many workgroups as the chip holds at once, and each takes work
// item after work item from a counter (kernels with short items lose more to the hand-over than they gain): XCD x
// serves the ids x, x + 8, x + 16, ... (which keeps a group's tiles on one L2, as above), in order, through counters[x];
// a workgroup whose own XCD has nothing left helps the others.  The loop ends for a workgroup once every counter has
// passed the end of its list, which every workgroup reaches.
//   thread 0:  take the next slot of the own XCD in advance (one atomic, its latency hidden behind an item) ...
__device__ inline unsigned queue_take_ahead(int32_t* counters, int xcd) { return atomicAdd((unsigned*)&counters[xcd], 1u); }
//   ... and turn it into a work id, or -1 when all lists are exhausted
__device__ inline int queue_resolve(int32_t* counters, int xcd, unsigned taken, unsigned per_xcd) {
    if (taken < per_xcd) return (int)(taken * N_XCD + xcd);
    for (int q = 1; q < N_XCD; q++) {
        const int x = (xcd + q) % N_XCD;
        const unsigned slot = atomicAdd((unsigned*)&counters[x], 1u);
        if (slot < per_xcd) return (int)(slot * N_XCD + x);
    }
    return -1;
}
// workgroups of `Kernel` (at `threads` threads, no dynamic LDS) that the current device holds at once
template <auto Kernel>
inline int resident_workgroups(int threads) {
    constexpr int MAX_DEVICES = 64;
    static std::atomic<int> cached[MAX_DEVICES];  // per device (0: not asked yet); the answer never changes
    int dev = 0, n_cu = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    const bool cacheable = dev >= 0 && dev < MAX_DEVICES;
    if (cacheable) {
        const int known = cached[dev].load(std::memory_order_relaxed);
        if (known > 0) return known;
    }
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 256;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, Kernel, threads, 0) != hipSuccess) return 256;
    const int n = n_cu * (per_cu > 0 ? per_cu : 1);
    if (cacheable) cached[dev].store(n, std::memory_order_relaxed);
    return n;
}
// fill `n` 32-bit words with zero (a kernel, so that a caller may capture the call in a HIP graph)
hipError_t launch_zero_words(void* ptr, size_t n_words, hipStream_t s);

}  // namespace hta
