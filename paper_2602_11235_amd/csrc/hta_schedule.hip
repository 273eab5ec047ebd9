// Work schedule of a jagged batch, built on the device from hist_len / n_targets (no host round trip).
//
// Under the hybrid mask (rules 1 and 3, Section 3.2.2) user b owns exactly the tiles
// (query rows) x (history keys): rows = L_b + T_b in a full layer, T_b in a target layer, keys = L_b
// (with real-time tokens, rule 2, their keys and rows count like history ones);
// nothing else is ever issued (the self key of a target row is a per-row term).  The attention
// kernels enumerate those tiles from (L_b, T_b) themselves; what the schedule adds is the ORDER of
// the users: workgroups are dispatched user-major, so listing users by decreasing tile count
// (rows x keys) starts the long-history users first and leaves the short ones to fill the tail.
#include "hta_common.h"

namespace hta {
namespace {

constexpr int SCHED_THREADS = 1024;
constexpr int RANK_SORT_MAX = 4096;   // exact, deterministic rank sort up to this many users
constexpr int N_BUCKETS = 2048;       // bucketed counting sort above it

// tiles a user owns: (query rows) x (keys that run through the tile loops: history, then real-time tokens)
__device__ inline float user_cost(const Params& p, int b) {
    const float L = (float)p.hist_len[b] + (p.rt_len ? (float)p.rt_len[b] : 0.f), T = (float)p.n_targets[b];
    return (p.layer == 0 ? L + T : T) * L;
}

// order[i] = user with the i-th largest cost; ties broken by user index, so the result is unique
__global__ __launch_bounds__(SCHED_THREADS) void schedule_rank_kernel(Params p, int32_t* counters, int32_t* order) {
    __shared__ float cost[RANK_SORT_MAX];
    const int B = p.batch;
    if (threadIdx.x < QUEUE_WORDS) counters[threadIdx.x] = 0;
    for (int b = threadIdx.x; b < B; b += SCHED_THREADS) cost[b] = user_cost(p, b);
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += SCHED_THREADS) {
        const float c = cost[b];
        int rank = 0;
        for (int o = 0; o < B; o++) {
            const float co = cost[o];  // same address for the whole wave: an LDS broadcast
            rank += (co > c || (co == c && o < b)) ? 1 : 0;
        }
        order[rank] = b;
    }
}

// Large batches: users fall into N_BUCKETS cost classes (by cost / max possible cost); classes are laid out
// by decreasing cost, users inside a class in arrival order of the atomics (any order is a valid schedule).
__global__ __launch_bounds__(SCHED_THREADS) void schedule_bucket_kernel(Params p, int32_t* counters, int32_t* order) {
    __shared__ int count[N_BUCKETS];
    __shared__ int start[N_BUCKETS];
    const int B = p.batch;
    if (threadIdx.x < QUEUE_WORDS) counters[threadIdx.x] = 0;
    const float keys_max = (float)max_lead_keys(p);
    const float rows_max = p.layer == 0 ? keys_max + (float)p.max_targets : (float)p.max_targets;
    const float inv = (float)(N_BUCKETS - 1) / fmaxf(rows_max * keys_max, 1.f);
    for (int i = threadIdx.x; i < N_BUCKETS; i += SCHED_THREADS) count[i] = 0;
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += SCHED_THREADS) {
        const int k = min(N_BUCKETS - 1, max(0, (int)(user_cost(p, b) * inv)));
        atomicAdd(&count[N_BUCKETS - 1 - k], 1);  // bucket 0 = most expensive class
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int i = 0; i < N_BUCKETS; i++) {
            start[i] = acc;
            acc += count[i];
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += SCHED_THREADS) {
        const int k = min(N_BUCKETS - 1, max(0, (int)(user_cost(p, b) * inv)));
        order[atomicAdd(&start[N_BUCKETS - 1 - k], 1)] = b;
    }
}

// Mask rule 2 (Section 3.2.2): a real-time token is visible only to tokens with later timestamps.  The real-time
// segment of a user is sorted by time, so the real-time keys a query sees are a prefix of it: those strictly earlier
// than the query.  lim[row] = hist_len + that prefix length = the number of leading K/V rows of the user the row
// attends to in the tile loops (its own key, when it is a real-time or target token, is a separate term).
__global__ __launch_bounds__(256) void rt_limits_kernel(Params p) {
    const int b = blockIdx.z;
    const int row = blockIdx.x * 256 + threadIdx.x;
    const int L = p.hist_len[b], R = p.rt_len[b], T = p.n_targets[b];
    const int n_rows = p.layer == 0 ? L + R + T : T;
    if (row >= n_rows) return;
    const int32_t* ts = p.ts + p.kv_off[b];
    const int32_t t = ts[p.layer == 0 ? row : L + R + row];
    int lo = 0, hi = R;  // first real-time token that is not strictly earlier than t
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (ts[L + mid] < t) lo = mid + 1; else hi = mid;
    }
    p.lim[(int64_t)p.q_off[b] + row] = L + lo;
}

// bf16 heads of 16 features ride the 32-wide matrix tiles zero-padded: rows [n][16] <-> [n][32] with the upper half
// zero (one thread per 16-byte chunk).  Zero features change no score and no gradient of the features that exist.
__global__ __launch_bounds__(256) void widen16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n_rows) {
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;  // chunk of the wide row
    if (id >= n_rows * 4) return;
    const int64_t row = id >> 2;
    const int c = (int)(id & 3);
    dst[id] = c < 2 ? src[row * 2 + c] : uint4{0u, 0u, 0u, 0u};
}
__global__ __launch_bounds__(256) void narrow16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n_rows) {
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;  // chunk of the narrow row
    if (id >= n_rows * 2) return;
    dst[id] = src[(id >> 1) * 4 + (id & 1)];
}

}  // namespace

hipError_t launch_widen16(const void* src, void* dst, int64_t n_rows, hipStream_t s) {
    if (n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(widen16_kernel, dim3((unsigned)((n_rows * 4 + 255) / 256)), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n_rows);
    return hipGetLastError();
}

hipError_t launch_narrow16(const void* src, void* dst, int64_t n_rows, hipStream_t s) {
    if (n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(narrow16_kernel, dim3((unsigned)((n_rows * 2 + 255) / 256)), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n_rows);
    return hipGetLastError();
}

hipError_t launch_rt_limits(const Params& p, hipStream_t s) {
    const int64_t rows = max_query_rows(p);
    if (p.batch <= 0 || rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(rt_limits_kernel, dim3((unsigned)((rows + 255) / 256), 1, (unsigned)p.batch), dim3(256), 0, s, p);
    return hipGetLastError();
}

size_t schedule_bytes(int32_t batch) {
    return QUEUE_WORDS * sizeof(int32_t) + ((((size_t)batch * sizeof(int32_t)) + 255) & ~(size_t)255);
}

hipError_t launch_schedule(const Params& p, void* region, hipStream_t s) {
    if (p.batch <= 0) return hipSuccess;
    int32_t* counters = (int32_t*)region;
    int32_t* order = schedule_order(region);
    if (p.batch <= RANK_SORT_MAX)
        hipLaunchKernelGGL(schedule_rank_kernel, dim3(1), dim3(SCHED_THREADS), 0, s, p, counters, order);
    else
        hipLaunchKernelGGL(schedule_bucket_kernel, dim3(1), dim3(SCHED_THREADS), 0, s, p, counters, order);
    return hipGetLastError();
}

}  // namespace hta
