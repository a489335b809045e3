// Kernel timer: device execution time of the kernels an entry point launches, for callers without a
// profiler.  Between lotts_timer_start and lotts_timer_stop every launch made by the calling host
// thread carries a pair of events of its own (hipExtLaunchKernel attaches them to the dispatch), so
// each pair reads that kernel's start and end on the device: no gap between commands is included.
#include <atomic>
#include <vector>

#include "lotts_common.h"

namespace lotts {

struct KernelTimer {
    std::vector<hipEvent_t> ev;  // 2 per launch; kept for the life of the thread and reused
    int capacity = 0;            // launches the running measurement may hold; 0 = timer off
    int used = 0;
    bool paused = false;
};
static thread_local KernelTimer g_timer;

static std::atomic<unsigned> g_word_tag{0};
unsigned next_word_tag() {
    unsigned tag = g_word_tag.fetch_add(1, std::memory_order_relaxed) + 1;
    if (tag == 0) tag = g_word_tag.fetch_add(1, std::memory_order_relaxed) + 1;  // 0 is what cleared words hold
    return tag;
}

bool timer_take(hipEvent_t* start, hipEvent_t* stop) {
    KernelTimer& t = g_timer;
    if (t.paused || t.used >= t.capacity) return false;
    *start = t.ev[2 * t.used];
    *stop = t.ev[2 * t.used + 1];
    ++t.used;
    return true;
}

}  // namespace lotts

extern "C" int lotts_timer_start(int32_t max_launches) {
    using namespace lotts;
    KernelTimer& t = g_timer;
    if (max_launches < 1 || max_launches > (1 << 20)) return LOTTS_ERR_SHAPE;
    while ((int)t.ev.size() < 2 * max_launches) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return LOTTS_ERR_LAUNCH;
        t.ev.push_back(e);
    }
    t.used = 0;
    t.paused = false;
    t.capacity = max_launches;
    return LOTTS_OK;
}

extern "C" int lotts_timer_pause(int32_t paused) {
    lotts::g_timer.paused = paused != 0;
    return LOTTS_OK;
}

extern "C" int lotts_timer_stop(int32_t* launches, float* ms) {
    using namespace lotts;
    KernelTimer& t = g_timer;
    if (!launches) return LOTTS_ERR_NULL;
    const int n = t.used;
    t.capacity = 0;  // off, whatever happens below
    t.used = 0;
    *launches = n;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(t.ev[2 * i + 1]) != hipSuccess) return LOTTS_ERR_LAUNCH;
        float v = 0.f;
        if (hipEventElapsedTime(&v, t.ev[2 * i], t.ev[2 * i + 1]) != hipSuccess) return LOTTS_ERR_LAUNCH;
        if (ms) ms[i] = v;
    }
    return LOTTS_OK;
}
