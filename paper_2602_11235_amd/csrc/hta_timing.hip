// Optional per-kernel timing with HIP events recorded on the caller's stream, around each kernel
// the library enqueues.  Off by default: when off, the hooks are two predictable branches.
#include "../../include/mtfm_hta.h"
#include "../../include/mtfm_hta_timing.h"
#include "hta_common.h"

#include <mutex>
#include <vector>

namespace hta {
namespace {

struct Ring {
    std::vector<hipEvent_t> begin, end;
    int next = 0;       // slot the next begin() uses
    int recorded = 0;   // complete (begin, end) pairs since the last read, capped at the ring size
    bool open = false;
};

std::mutex g_mu;
bool g_on = false;
Ring g_ring[MTFM_HTA_N_KERNELS];

void destroy_all() {
    for (Ring& r : g_ring) {
        for (hipEvent_t e : r.begin) (void)hipEventDestroy(e);
        for (hipEvent_t e : r.end) (void)hipEventDestroy(e);
        r = Ring();
    }
}

}  // namespace

void timing_begin(int kind, hipStream_t s) {
    if (!g_on) return;
    std::lock_guard<std::mutex> lock(g_mu);
    Ring& r = g_ring[kind];
    if (r.begin.empty()) return;
    (void)hipEventRecord(r.begin[r.next], s);
    r.open = true;
}

void timing_end(int kind, hipStream_t s) {
    if (!g_on) return;
    std::lock_guard<std::mutex> lock(g_mu);
    Ring& r = g_ring[kind];
    if (r.begin.empty() || !r.open) return;
    (void)hipEventRecord(r.end[r.next], s);
    r.open = false;
    r.next = (r.next + 1) % (int)r.begin.size();
    if (r.recorded < (int)r.begin.size()) r.recorded++;
}

}  // namespace hta

extern "C" {

int mtfm_hta_timing_enable(int slots) {
    std::lock_guard<std::mutex> lock(hta::g_mu);
    hta::destroy_all();
    hta::g_on = false;
    if (slots <= 0) return MTFM_HTA_OK;
    if (slots > 4096) return MTFM_HTA_ERR_INVALID_ARG;
    for (hta::Ring& r : hta::g_ring) {
        r.begin.resize(slots);
        r.end.resize(slots);
        for (int i = 0; i < slots; i++) {
            if (hipEventCreate(&r.begin[i]) != hipSuccess || hipEventCreate(&r.end[i]) != hipSuccess) {
                r.begin.resize(i);  // events past i were never created
                r.end.resize(i);
                hta::destroy_all();
                return MTFM_HTA_ERR_LAUNCH;
            }
        }
    }
    hta::g_on = true;
    return MTFM_HTA_OK;
}

int mtfm_hta_timing_read(int kernel, float* ms, int capacity) {
    if (kernel < 0 || kernel >= MTFM_HTA_N_KERNELS || capacity < 0 || (capacity > 0 && !ms)) return MTFM_HTA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(hta::g_mu);
    hta::Ring& r = hta::g_ring[kernel];
    const int size = (int)r.begin.size();
    int n = r.recorded < capacity ? r.recorded : capacity;
    int written = 0;
    for (int i = 0; i < n; i++) {
        const int slot = ((r.next - r.recorded + i) % size + size) % size;
        if (hipEventSynchronize(r.end[slot]) != hipSuccess) break;
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.begin[slot], r.end[slot]) != hipSuccess) break;
        ms[written++] = t;
    }
    r.recorded = 0;
    return written;
}

}  // extern "C"
