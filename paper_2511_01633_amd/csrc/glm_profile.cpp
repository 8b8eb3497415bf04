// Optional per-kernel timing with HIP events recorded on the stream each kernel is launched on.
// Off by default: the hot calls then record nothing.
#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "glm_internal.h"

namespace glm {

namespace {
struct Sample { hipEvent_t start, stop; int id; };
std::mutex g_mu;
std::atomic<bool> g_enabled{false};       // read by every launch: no lock on the hot path
std::vector<Sample> g_samples;
}  // namespace

ProfileScope::ProfileScope(int id, hipStream_t st) : st_(st), id_(id) {
    active_ = g_enabled.load(std::memory_order_relaxed);
    if (!active_) return;
    if (hipEventCreate(&start_) != hipSuccess || hipEventCreate(&stop_) != hipSuccess ||
        hipEventRecord(start_, st_) != hipSuccess)
        active_ = false;
}

ProfileScope::~ProfileScope() {
    if (!active_) return;
    if (hipEventRecord(stop_, st_) != hipSuccess) return;
    std::lock_guard<std::mutex> lk(g_mu);
    g_samples.push_back({start_, stop_, id_});
}

}  // namespace glm

using namespace glm;

extern "C" {

int glm_profile_enable(int on) {
    g_enabled.store(on != 0, std::memory_order_relaxed);
    return GLM_OK;
}

int glm_profile_reset(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    for (Sample &s : g_samples) { (void)hipEventDestroy(s.start); (void)hipEventDestroy(s.stop); }
    g_samples.clear();
    return GLM_OK;
}

int glm_profile_read_stats(int kernel_id, double *total_ms, int64_t *launches, double *min_ms, double *median_ms) {
    std::lock_guard<std::mutex> lk(g_mu);
    std::vector<float> t_all;
    double ms = 0.0;
    for (Sample &s : g_samples) {
        if (s.id != kernel_id) continue;
        hipError_t e = hipEventSynchronize(s.stop);
        float t = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&t, s.start, s.stop);
        if (e != hipSuccess) return set_hip_error(e);
        ms += t;
        t_all.push_back(t);
    }
    std::sort(t_all.begin(), t_all.end());
    const size_t n = t_all.size();
    if (total_ms) *total_ms = ms;
    if (launches) *launches = (int64_t)n;
    if (min_ms) *min_ms = n ? t_all[0] : 0.0;
    if (median_ms) *median_ms = n ? 0.5 * (t_all[(n - 1) / 2] + t_all[n / 2]) : 0.0;
    return GLM_OK;
}

int glm_profile_read(int kernel_id, double *total_ms, int64_t *launches) {
    return glm_profile_read_stats(kernel_id, total_ms, launches, nullptr, nullptr);
}

}  // extern "C"
