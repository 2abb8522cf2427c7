// Bandwidth calibration kernels: a plain copy and a plain fill over a byte range.  They are not
// part of the method; the benchmark uses them to state what this GPU's memory system delivers to
// the simplest possible kernel (the practical ceiling next to the published HBM peak), and profiler
// byte counters are scaled by what they read for a copy of known size.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.hpp"

namespace aura {

typedef uint32_t cal_u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCalThreads = 256;
constexpr int kCalUnroll = 4;   // 16-byte accesses per thread and loop trip

__global__ __launch_bounds__(kCalThreads) void k_calibration_copy(cal_u32x4* __restrict__ dst, const cal_u32x4* __restrict__ src,
                                                                  long long n_vec) {
  const long long stride = (long long)gridDim.x * kCalThreads * kCalUnroll;
  for (long long base = (long long)blockIdx.x * kCalThreads * kCalUnroll + threadIdx.x; base < n_vec; base += stride) {
    cal_u32x4 v[kCalUnroll];
#pragma unroll
    for (int u = 0; u < kCalUnroll; ++u) {
      const long long i = base + (long long)u * kCalThreads;
      if (i < n_vec) v[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < kCalUnroll; ++u) {
      const long long i = base + (long long)u * kCalThreads;
      if (i < n_vec) __builtin_nontemporal_store(v[u], dst + i);
    }
  }
}

__global__ __launch_bounds__(kCalThreads) void k_calibration_fill(cal_u32x4* __restrict__ dst, uint32_t value, long long n_vec) {
  const long long stride = (long long)gridDim.x * kCalThreads * kCalUnroll;
  const cal_u32x4 v = {value, value, value, value};
  for (long long base = (long long)blockIdx.x * kCalThreads * kCalUnroll + threadIdx.x; base < n_vec; base += stride) {
#pragma unroll
    for (int u = 0; u < kCalUnroll; ++u) {
      const long long i = base + (long long)u * kCalThreads;
      if (i < n_vec) __builtin_nontemporal_store(v, dst + i);
    }
  }
}

static int calibration_grid(long long n_vec) {
  const long long per_block = (long long)kCalThreads * kCalUnroll;
  const long long need = (n_vec + per_block - 1) / per_block;
  const long long cap = 256 * 16;   // 16 workgroups per compute unit
  return (int)(need < 1 ? 1 : (need > cap ? cap : need));
}

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const long long n_vec = (long long)(bytes / 16);
  hipLaunchKernelGGL(k_calibration_copy, dim3(calibration_grid(n_vec)), dim3(kCalThreads), 0, stream,
                     static_cast<cal_u32x4*>(dst), static_cast<const cal_u32x4*>(src), n_vec);
  return hipGetLastError();
}

hipError_t launch_calibration_fill(void* dst, size_t bytes, uint32_t value, hipStream_t stream) {
  const long long n_vec = (long long)(bytes / 16);
  hipLaunchKernelGGL(k_calibration_fill, dim3(calibration_grid(n_vec)), dim3(kCalThreads), 0, stream,
                     static_cast<cal_u32x4*>(dst), value, n_vec);
  return hipGetLastError();
}

}  // namespace aura
