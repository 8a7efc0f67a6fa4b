// Optional per-kernel timing (diagnostics for the benchmark: off by default, not thread-safe).  Each
// timed launch carries a start and a stop event that receive the kernel's own begin and end stamps.
#include <vector>

#include "ssd_internal.h"

namespace ssdk {
namespace {

struct Rec {
    int kid;
    hipEvent_t a, b;
};

bool g_on = false;
int g_only = -1;  // >= 0: record this kernel id only
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
const char* const g_names[K_COUNT] = {
    "cumsum", "cb", "chunk_state", "state_scan_fwd", "chunk_out", "dstate_local", "state_scan_bwd", "bwd_main",
    "ddt_finalize", "param_reduce", "dG", "dBC", "fill", "copy",
    "mfma_cb", "mfma_chunk_state", "mfma_chunk_out", "mfma_dstate_local", "mfma_bwd_main", "mfma_dG", "mfma_dBC", "mfma_dBC_final", "mfma_bwd_trio", "mfma_prep_cb", "mfma_final_ddt"};

hipEvent_t take_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

}  // namespace

bool prof_events(int kid, hipEvent_t* start, hipEvent_t* stop) {
    if (!g_on || (g_only >= 0 && kid != g_only)) return false;
    Rec r{kid, take_event(), take_event()};
    if (!r.a || !r.b) return false;
    g_recs.push_back(r);
    *start = r.a;
    *stop = r.b;
    return true;
}

}  // namespace ssdk

using namespace ssdk;

extern "C" int ssd_prof_enable(int32_t on) {
    for (Rec& r : g_recs) {
        (void)hipEventSynchronize(r.b);
        g_pool.push_back(r.a);
        g_pool.push_back(r.b);
    }
    g_recs.clear();
    g_on = on != 0;
    g_only = on >= 2 ? on - 2 : -1;
    if (g_only >= K_COUNT) return SSD_ERR_ARG;
    return SSD_OK;
}

extern "C" int ssd_prof_read(int32_t kernel_id, double* total_ms, int64_t* launches) {
    if (!total_ms || !launches) return SSD_ERR_NULL;
    if (kernel_id < 0 || kernel_id >= K_COUNT) return SSD_ERR_ARG;
    double t = 0.0;
    int64_t n = 0;
    for (Rec& r : g_recs) {
        if (r.kid != kernel_id) continue;
        if (hipEventSynchronize(r.b) != hipSuccess) return SSD_ERR_LAUNCH;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return SSD_ERR_LAUNCH;
        t += ms;
        ++n;
    }
    *total_ms = t;
    *launches = n;
    return SSD_OK;
}

extern "C" const char* ssd_prof_kernel_name(int32_t kernel_id) {
    return (kernel_id >= 0 && kernel_id < K_COUNT) ? g_names[kernel_id] : nullptr;
}
