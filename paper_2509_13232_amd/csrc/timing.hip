// Per-kernel timing instrumentation: pairs of HIP events recorded around the
// launches of each kernel class, read back (and reset) on request.
#include "timing.hpp"

#include <mutex>
#include <utility>
#include <vector>

namespace spo {

static std::mutex g_mu;
static bool g_on = false;
static std::vector<std::pair<hipEvent_t, hipEvent_t>> g_pairs[kTimeClasses];
static hipEvent_t g_open[kTimeClasses];
static std::vector<hipEvent_t> g_pool;  // events that have been read: reused, so that steady-state timing creates none

bool timing_enabled() { return g_on; }

static bool take_event(hipEvent_t *e) {
    if (!g_pool.empty()) {
        *e = g_pool.back();
        g_pool.pop_back();
        return true;
    }
    return hipEventCreate(e) == hipSuccess;
}

void timing_begin(int cls, hipStream_t s) {
    std::lock_guard<std::mutex> lk(g_mu);
    hipEvent_t a;
    if (!take_event(&a)) return;
    (void)hipEventRecord(a, s);
    g_open[cls] = a;
}

void timing_end(int cls, hipStream_t s) {
    std::lock_guard<std::mutex> lk(g_mu);
    hipEvent_t b;
    if (!g_open[cls] || !take_event(&b)) return;
    (void)hipEventRecord(b, s);
    g_pairs[cls].emplace_back(g_open[cls], b);
    g_open[cls] = nullptr;
}

}  // namespace spo

using namespace spo;

extern "C" int spo_kernel_timing_enable(int enable) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = enable != 0;
    return SPO_OK;
}

extern "C" int spo_kernel_timing_read(float *ms, int32_t *launches) {
    if (!ms || !launches) return SPO_ENULL;
    std::lock_guard<std::mutex> lk(g_mu);
    int rc = SPO_OK;
    for (int c = 0; c < kTimeClasses; ++c) {
        float total = 0.0f;
        for (auto &p : g_pairs[c]) {
            float t = 0.0f;
            if (hipEventSynchronize(p.second) != hipSuccess || hipEventElapsedTime(&t, p.first, p.second) != hipSuccess)
                rc = SPO_EHIP;
            total += t;
            g_pool.push_back(p.first);
            g_pool.push_back(p.second);
        }
        ms[c] = total;
        launches[c] = static_cast<int32_t>(g_pairs[c].size());
        g_pairs[c].clear();
    }
    return rc;
}
