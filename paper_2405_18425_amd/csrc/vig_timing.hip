// Per-kernel HIP-event timing behind vig_timing_enable / vig_timing_collect.
#include <vector>

#include "../../include/vig_bigla.h"
#include "vig_timing.hpp"

namespace vig {

namespace {

struct Record {
    int id;
    hipEvent_t start, stop;
};

struct TimingState {
    bool on = false;
    std::vector<Record> pool;  // events are created once and reused
    size_t used = 0;
};

thread_local TimingState g_timing;

}  // namespace

LaunchTimer::LaunchTimer(KernelId id, hipStream_t stream) : slot_(-1), stream_(stream)
{
    TimingState &t = g_timing;
    if (!t.on) return;
    if (t.used == t.pool.size()) {
        Record r;
        r.id = id;
        if (hipEventCreate(&r.start) != hipSuccess) return;
        if (hipEventCreate(&r.stop) != hipSuccess) {
            (void)hipEventDestroy(r.start);
            return;
        }
        t.pool.push_back(r);
    }
    slot_ = int(t.used++);
    t.pool[slot_].id = id;
    (void)hipEventRecord(t.pool[slot_].start, stream_);
}

LaunchTimer::~LaunchTimer()
{
    if (slot_ >= 0) (void)hipEventRecord(g_timing.pool[slot_].stop, stream_);
}

}  // namespace vig

extern "C" {

int vig_timing_enable(int on)
{
    vig::g_timing.on = on != 0;
    vig::g_timing.used = 0;
    return VIG_OK;
}

int vig_timing_collect(int kernel, double *total_ms, long *launches)
{
    if (!total_ms || !launches) return VIG_ERR_NULL;
    if (kernel < 0 || kernel >= vig::kKernelCount) return VIG_ERR_SHAPE;
    double sum = 0.0;
    long n = 0;
    for (size_t i = 0; i < vig::g_timing.used; ++i) {
        const vig::Record &r = vig::g_timing.pool[i];
        if (r.id != kernel) continue;
        if (hipEventSynchronize(r.stop) != hipSuccess) return VIG_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return VIG_ERR_HIP;
        sum += ms;
        ++n;
    }
    *total_ms = sum;
    *launches = n;
    return VIG_OK;
}

}  // extern "C"
