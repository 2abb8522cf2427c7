// aura_material_scores_static: aura_material_scores for callers that cannot allocate device memory or pass a
// workspace (code under stream capture, serving loops with a fixed memory plan, harnesses that forbid allocation).
// The scratch that the scoring kernels need - the text embeddings split into two bf16 terms in operand order - lives in
// a fixed array in the library's own device image instead of a caller's workspace.  Every GPU the library runs on holds
// its own copy of that array until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/aura_fuse.h"
#include "abi_util.hpp"
#include "launch.hpp"

namespace {

constexpr size_t kScratchBytes = AURA_STATIC_SCRATCH_BYTES;

// Device memory owned by the library.  In host code this name only stands for the symbol: the address that kernels
// and copies need comes from hipGetSymbolAddress, once per device (scratch_of_current_device).
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// The address of the current device's copy of `scratch`.
hipError_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

aura_status_t aura_material_scores_static(const float* fused, int64_t N, int32_t D, const void* temb, int32_t temb_dtype,
                                          int32_t K, const float* y, int32_t P, const aura_params_t* params, float* scores,
                                          float* prop, int32_t* label, void* stream) {
  if (!params || !temb) return AURA_ERR_NULL;
  if (N < 0 || D < 1 || K < 1 || P < 0) return AURA_ERR_SHAPE;
  if (temb_dtype != AURA_F32 && temb_dtype != AURA_BF16 && temb_dtype != AURA_F16) return AURA_ERR_DTYPE;
  if (prop && (!y || P < 1)) return AURA_ERR_NULL;
  if (!(params->temperature > 0.0f)) return AURA_ERR_SHAPE;
  if (K > 128 || P > 8) return AURA_ERR_UNSUPPORTED;
  if (aura::scores_workspace_bytes(D, K) > kScratchBytes) return AURA_ERR_UNSUPPORTED;   // beyond the fixed scratch
  if (N == 0) return AURA_OK;
  if (!fused || !scores) return AURA_ERR_NULL;
  void* ws = nullptr;
  const aura_status_t s = aura::hip_status(scratch_of_current_device(&ws));
  if (s != AURA_OK) return s;
  // The array holds the fp32 copy of 16-bit embeddings (behind the split embeddings) and the split embeddings; both
  // are rewritten in full by the first launches of the call before anything reads them: nothing of an earlier call
  // is seen.
  const hipStream_t st = static_cast<hipStream_t>(stream);
  const float* t32 = static_cast<const float*>(temb);
  if (temb_dtype != AURA_F32) {
    float* copy = reinterpret_cast<float*>(static_cast<char*>(ws) + aura::scores_split_bytes(D, K));
    const aura_status_t sw = aura::hip_status(aura::launch_widen_embeddings(temb, temb_dtype, (long long)K * D, copy, st));
    if (sw != AURA_OK) return sw;
    t32 = copy;
  }
  return aura::hip_status(aura::launch_material_scores(fused, N, D, t32, K, y, P, params->temperature, scores, prop, label,
                                                       ws, st, (params->flags & AURA_UNSEEN_ZERO) ? 1 : 0));
}

}  // extern "C"
