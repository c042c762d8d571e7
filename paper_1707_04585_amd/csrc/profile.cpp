// Optional per-kernel timing with HIP events, for roofline reports.
//
// While enabled, every kernel launch of the library carries a pair of events
// that the dispatch itself stamps with the kernel's start and end times on the
// stream it runs on (hipExtLaunchKernelGGL), so the elapsed time between them
// is the kernel's own duration.  The events come from a pool that grows on
// demand (host allocations only; no device memory).  Profiling perturbs the
// gaps between kernels and is meant for a separate pass.
#include <mutex>
#include <vector>

#include "kernels.h"

namespace rvn {
namespace {

struct Mark {
    int id;
    double bytes, flops;
    hipEvent_t start, stop;
};

std::mutex g_mu;
bool g_on = false;
std::vector<Mark> g_marks;
std::vector<hipEvent_t> g_pool;

hipEvent_t take_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

const char *const kNames[K_COUNT] = {
    "bn_stats_k", "clear_counters_k", "conv_fwd", "conv_dgrad",
    "conv_wgrad", "wgrad_reduce_k", "bn_bwd_reduce_k", "bn_bwd_apply_k", "prep_filter_k", "conv_dgrad_wgrad",
    "resample2_k", "fixed_point_k", "stem_k", "splitk_reduce_k",
};

}  // namespace

const char *kernel_name(int id) { return id >= 0 && id < K_COUNT ? kNames[id] : "?"; }

bool profile_enabled() { return g_on; }

void profile_new_mark(int id, double bytes, double flops, hipEvent_t *start, hipEvent_t *stop) {
    std::lock_guard<std::mutex> lk(g_mu);
    Mark m{id, bytes, flops, take_event(), take_event()};
    g_marks.push_back(m);
    *start = m.start;
    *stop = m.stop;
}

}  // namespace rvn

using namespace rvn;

extern "C" {

int revnet_profile_begin(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    for (Mark &m : g_marks) {
        g_pool.push_back(m.start);
        g_pool.push_back(m.stop);
    }
    g_marks.clear();
    g_on = true;
    return RVN_OK;
}

int revnet_profile_end(rvn_kernel_stat *stats, int32_t max_stats, int32_t *n_stats) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = false;
    rvn_kernel_stat acc[K_COUNT] = {};
    hipError_t err = hipSuccess;
    for (Mark &m : g_marks) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(m.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, m.start, m.stop);
        if (e != hipSuccess) err = e;
        acc[m.id].launches += 1;
        acc[m.id].total_ms += ms;
        acc[m.id].algorithmic_bytes += m.bytes;
        acc[m.id].flops += m.flops;
        g_pool.push_back(m.start);
        g_pool.push_back(m.stop);
    }
    g_marks.clear();
    int32_t n = 0;
    for (int id = 0; id < K_COUNT; ++id) {
        if (!acc[id].launches) continue;
        if (stats && n < max_stats) {
            acc[id].name = kernel_name(id);
            stats[n] = acc[id];
        }
        ++n;
    }
    if (n_stats) *n_stats = n;
    return err == hipSuccess ? RVN_OK : RVN_ERR_HIP;
}

}  // extern "C"
