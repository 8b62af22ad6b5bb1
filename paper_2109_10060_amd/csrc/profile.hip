// Optional per-kernel timing: while recording, every kernel launcher brackets its launch
// with a pair of HIP events on the launch stream; ds_profile_read sums the elapsed
// times per kernel class.  Off by default; costs nothing when off.  Recording can be
// paused and resumed (records accumulate) so that a caller samples some of its steps.
// The record list is guarded by one mutex, so launchers on several host threads may record at once; the
// records then interleave in the order the threads took the lock.
#include <atomic>
#include <mutex>
#include <vector>

#include "common.h"

namespace {
struct Rec {
    hipEvent_t a, b;
    int kind;
};
std::atomic<bool> g_on{false};
thread_local int t_paused = 0;   // entry points that must not allocate pause recording on their own thread only
std::mutex g_mu;                 // guards g_pool and g_used
std::vector<Rec> g_pool;         // events are created once and reused
size_t g_used = 0;
}  // namespace

ProfScope::ProfScope(int kind, hipStream_t stream) : rec(-1), s(stream) {
    if (!g_on.load(std::memory_order_relaxed) || t_paused) return;
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_used == g_pool.size()) {
        Rec r;
        if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
        r.kind = kind;
        g_pool.push_back(r);
    }
    rec = (int)g_used++;
    g_pool[rec].kind = kind;
    (void)hipEventRecord(g_pool[rec].a, s);
}

ProfScope::~ProfScope() {
    if (rec < 0) return;
    std::lock_guard<std::mutex> lock(g_mu);
    if ((size_t)rec < g_pool.size()) (void)hipEventRecord(g_pool[rec].b, s);
}

// recording creates HIP events on first use; entry points that must not allocate switch it off for their duration
ProfPause::ProfPause() : was(t_paused != 0) { ++t_paused; }
ProfPause::~ProfPause() { --t_paused; }

extern "C" int32_t ds_profile_enable(int32_t on) {
    g_on.store(on != 0);
    return DS_OK;
}

extern "C" int32_t ds_profile_reset(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    g_used = 0;
    return DS_OK;
}

extern "C" int32_t ds_profile_read(int32_t kind, double* total_ms, int64_t* launches) {
    if (kind < 0 || kind >= DS_K_COUNT || !total_ms || !launches) DS_FAIL(DS_EINVAL, "ds_profile_read: bad argument");
    double t = 0.0;
    int64_t n = 0;
    std::lock_guard<std::mutex> lock(g_mu);
    for (size_t i = 0; i < g_used; ++i) {
        if (g_pool[i].kind != kind) continue;
        if (hipEventSynchronize(g_pool[i].b) != hipSuccess) DS_FAIL(DS_EHIP, "ds_profile_read: event sync failed");
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_pool[i].a, g_pool[i].b) != hipSuccess) DS_FAIL(DS_EHIP, "ds_profile_read: elapsed time failed");
        t += ms;
        ++n;
    }
    *total_ms = t;
    *launches = n;
    return DS_OK;
}

extern "C" int32_t ds_profile_launches(int32_t* kinds, float* ms, int64_t capacity, int64_t* count) {
    if (!count || capacity < 0 || (capacity > 0 && (!kinds || !ms))) DS_FAIL(DS_EINVAL, "ds_profile_launches: bad argument");
    std::lock_guard<std::mutex> lock(g_mu);
    *count = (int64_t)g_used;
    for (size_t i = 0; i < g_used && (int64_t)i < capacity; ++i) {
        if (hipEventSynchronize(g_pool[i].b) != hipSuccess) DS_FAIL(DS_EHIP, "ds_profile_launches: event sync failed");
        float t = 0.f;
        if (hipEventElapsedTime(&t, g_pool[i].a, g_pool[i].b) != hipSuccess) DS_FAIL(DS_EHIP, "ds_profile_launches: elapsed time failed");
        kinds[i] = g_pool[i].kind;
        ms[i] = t;
    }
    return DS_OK;
}
