// Per-kernel HIP-event timing behind vig_timing_enable / vig_timing_collect.
#include <vector>

#include "../../include/vig_bigla.h"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

struct Record {
    int id;
    hipEvent_t start, stop;
};

// Event pairs are created by vig_timing_enable(1), never inside a launch: once the pool is used
// up, further launches go unrecorded.
constexpr size_t kPoolRecords = 16384;

struct TimingState {
    bool on = false;
    std::vector<Record> pool;
    size_t used = 0;
};

thread_local TimingState g_timing;

}  // namespace

LaunchTimer::LaunchTimer(KernelId id, hipStream_t stream) : slot_(-1), stream_(stream)
{
    TimingState &t = g_timing;
    if (!t.on || t.used == t.pool.size()) return;
    // a stream under graph capture is left alone: event records would become nodes of the graph
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess || capture != hipStreamCaptureStatusNone) return;
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
    vig::TimingState &t = vig::g_timing;
    t.on = on != 0;
    t.used = 0;
    if (t.on && t.pool.size() < vig::kPoolRecords) {
        t.pool.reserve(vig::kPoolRecords);
        while (t.pool.size() < vig::kPoolRecords) {
            vig::Record r;
            r.id = -1;
            if (hipEventCreate(&r.start) != hipSuccess) return VIG_ERR_HIP;
            if (hipEventCreate(&r.stop) != hipSuccess) {
                (void)hipEventDestroy(r.start);
                return VIG_ERR_HIP;
            }
            t.pool.push_back(r);
        }
    }
    return VIG_OK;
}

int vig_measure_alias_slabs(int on)
{
    return vig::bigla_chunk_set_alias(on != 0 ? 1 : 0) == hipSuccess ? VIG_OK : VIG_ERR_HIP;
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
