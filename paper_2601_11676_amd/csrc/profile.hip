// Benchmark aid: a HIP event pair attached to the dispatch of the FFN's dominant kernel
// (the gate/up projection streams two thirds of the surviving groups' weight bytes).
// Inactive unless halo_profile_begin was called; never use while a stream is being
// captured into a graph.
#include "../../include/halo.h"

#include <mutex>
#include <string>
#include <vector>

#include "kernels.hpp"

namespace halo {
namespace {
struct Timer {
    std::mutex mu;
    bool active = false;
    std::vector<hipEvent_t> start, stop;
    size_t used = 0;
    int every = 1;          // time one launch in `every`
    long long seen = 0;     // eligible launches since begin
    std::string name;
} g_timer;
}  // namespace

bool timer_acquire(hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_timer.active) return false;
    std::lock_guard<std::mutex> lk(g_timer.mu);
    if (!g_timer.active || g_timer.used >= g_timer.start.size()) return false;
    if (g_timer.seen++ % g_timer.every != 0) return false;
    *start = g_timer.start[g_timer.used];
    *stop = g_timer.stop[g_timer.used];
    return true;
}

void timer_commit(const char *kernel_name)
{
    std::lock_guard<std::mutex> lk(g_timer.mu);
    if (!g_timer.active) return;
    ++g_timer.used;
    g_timer.name = kernel_name;
}

}  // namespace halo

extern "C" {

int halo_profile_begin(int32_t max_launches, int32_t every)
{
    using namespace halo;
    if (max_launches < 1 || max_launches > (1 << 20) || every < 1) return HALO_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_timer.mu);
    if (g_timer.active) return HALO_ERR_ARG;
    g_timer.start.assign((size_t)max_launches, nullptr);
    g_timer.stop.assign((size_t)max_launches, nullptr);
    for (int i = 0; i < max_launches; ++i) {
        if (hipEventCreate(&g_timer.start[i]) != hipSuccess || hipEventCreate(&g_timer.stop[i]) != hipSuccess)
            return HALO_ERR_HIP;
    }
    g_timer.used = 0;
    g_timer.every = every;
    g_timer.seen = 0;
    g_timer.name.clear();
    g_timer.active = true;
    return HALO_OK;
}

int halo_profile_end(double *total_ms, int64_t *launches, char *kernel_name, int32_t name_cap)
{
    using namespace halo;
    std::lock_guard<std::mutex> lk(g_timer.mu);
    if (!g_timer.active) return HALO_ERR_ARG;
    g_timer.active = false;
    double sum = 0.0;
    int rc = HALO_OK;
    for (size_t i = 0; i < g_timer.used; ++i) {
        float ms = 0.0f;
        if (hipEventSynchronize(g_timer.stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_timer.start[i], g_timer.stop[i]) != hipSuccess)
            rc = HALO_ERR_HIP;
        sum += ms;
    }
    if (total_ms) *total_ms = sum;
    if (launches) *launches = (int64_t)g_timer.used;
    if (kernel_name && name_cap > 0) {
        size_t n = g_timer.name.size() < (size_t)name_cap - 1 ? g_timer.name.size() : (size_t)name_cap - 1;
        g_timer.name.copy(kernel_name, n);
        kernel_name[n] = 0;
    }
    for (size_t i = 0; i < g_timer.start.size(); ++i) {
        if (g_timer.start[i]) (void)hipEventDestroy(g_timer.start[i]);
        if (g_timer.stop[i]) (void)hipEventDestroy(g_timer.stop[i]);
    }
    g_timer.start.clear();
    g_timer.stop.clear();
    g_timer.used = 0;
    return rc;
}

}  // extern "C"
