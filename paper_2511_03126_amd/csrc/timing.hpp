// The one-shot timing request behind aura_time_next_fusion: a pair of events that the next launch of a
// fusion kernel (made by the same host thread) records on its stream right before and right after itself.
#pragma once

#include <hip/hip_runtime.h>

namespace aura {

struct TimingRequest {
  hipEvent_t start = nullptr, stop = nullptr;
};

// Returns this thread's pending request and clears it (both events null when there is none).
TimingRequest take_timing_request();

}  // namespace aura
