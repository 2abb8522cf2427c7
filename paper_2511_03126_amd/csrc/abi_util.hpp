// Small helpers shared by the files that implement C ABI entry points.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/aura_fuse.h"

namespace aura {

// AURA_OK for hipSuccess; otherwise remembers the error for aura_last_hip_error() (per host thread) and returns
// AURA_ERR_HIP.
aura_status_t hip_status(hipError_t e);

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace aura
