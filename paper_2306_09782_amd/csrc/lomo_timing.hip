// Optional per-kernel timing with HIP events recorded on the launch stream.  Off by default;
// when on, every launch of a timed kernel family is bracketed by two events from a reusable pool.
#include "lomo.h"
#include "lomo_kernels.h"

#include <mutex>
#include <utility>
#include <vector>

namespace lomo {

namespace {
struct Pool {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev;
    size_t used = 0;
};
std::mutex g_mu;
bool g_on = false;
Pool g_pool[LOMO_KERNEL_FAMILIES];
constexpr size_t kMaxEventsPerFamily = 1u << 16;
}  // namespace

// Hands out the next (start, stop) event pair of a family for a launch that records them as part
// of its own dispatch; the pair counts as used.  False when timing is off.
bool timing_slot(int family, hipEvent_t* start, hipEvent_t* stop) {
    if (!g_on) return false;
    std::lock_guard<std::mutex> lk(g_mu);
    Pool& p = g_pool[family];
    if (p.used == p.ev.size()) {
        if (p.ev.size() >= kMaxEventsPerFamily) return false;
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return false;
        if (hipEventCreate(&b) != hipSuccess) {
            (void)hipEventDestroy(a);
            return false;
        }
        p.ev.emplace_back(a, b);
    }
    *start = p.ev[p.used].first;
    *stop = p.ev[p.used].second;
    p.used++;
    return true;
}

bool timing_begin(int family, hipStream_t st) {
    if (!g_on) return false;
    std::lock_guard<std::mutex> lk(g_mu);
    Pool& p = g_pool[family];
    if (p.used == p.ev.size()) {
        if (p.ev.size() >= kMaxEventsPerFamily) return false;
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return false;
        if (hipEventCreate(&b) != hipSuccess) {
            (void)hipEventDestroy(a);
            return false;
        }
        p.ev.emplace_back(a, b);
    }
    return hipEventRecord(p.ev[p.used].first, st) == hipSuccess;
}

void timing_end(int family, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_mu);
    Pool& p = g_pool[family];
    if (hipEventRecord(p.ev[p.used].second, st) == hipSuccess) p.used++;
}

}  // namespace lomo

extern "C" {

lomo_status lomo_timing_enable(int on) {
    std::lock_guard<std::mutex> lk(lomo::g_mu);
    lomo::g_on = on != 0;
    for (auto& p : lomo::g_pool) p.used = 0;
    return LOMO_OK;
}

lomo_status lomo_timing_read(int family, double* total_ms, int64_t* launches) {
    if (family < 0 || family >= LOMO_KERNEL_FAMILIES) return LOMO_ERR_SHAPE;
    if (!total_ms || !launches) return LOMO_ERR_NULL;
    std::lock_guard<std::mutex> lk(lomo::g_mu);
    lomo::Pool& p = lomo::g_pool[family];
    double sum = 0.0;
    for (size_t i = 0; i < p.used; ++i) {
        if (hipEventSynchronize(p.ev[i].second) != hipSuccess) return LOMO_ERR_LAUNCH;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.ev[i].first, p.ev[i].second) != hipSuccess) return LOMO_ERR_LAUNCH;
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int64_t)p.used;
    return LOMO_OK;
}

}  // extern "C"
