// Optional per-kernel timing with HIP events, recorded on the stream each kernel is launched on.
// Off by default (a launch then costs one thread-local flag test).
#pragma once

#include <hip/hip_runtime.h>

namespace vig {

enum KernelId {
    kKernelSegmentState = 0,
    kKernelGateLowrank = 1,
    kKernelSegmentOut = 2,
    kKernelRecurrent = 3,
    kKernelLocalityGate = 4,
    kKernelSegmentOutGeneral = 5,
    kKernelGateProducer = 6,
    kKernelSlab = 7,
    kKernelBackward = 8,
    kKernelCount = 9
};

// Brackets one launch when timing is enabled on the calling thread.
class LaunchTimer {
  public:
    LaunchTimer(KernelId id, hipStream_t stream);
    ~LaunchTimer();

  private:
    int slot_;
    hipStream_t stream_;
};

}  // namespace vig
