// Epilogue shared by the scoring kernels (Sec. 3.4.1): from the similarities omega of one point, held as
// matrix-core accumulators, to the stored scores, the arg-max label and the kernel regression of Eq. 4.
#pragma once

#include "aura_device.hpp"

namespace aura {

typedef float scores_f32x4 __attribute__((ext_vector_type(4)));
typedef float scores_f32x16 __attribute__((ext_vector_type(16)));

constexpr int kScoreTileM = 32;   // materials per matrix-core tile
constexpr int kScoreMaxP = 8;
constexpr int kScoreMaxK = 128;

// Lane l = 32 g + (point within the wave's 32): accumulator element r of tile mt is the similarity of the
// lane's point to material mt*32 + 8*(r/4) + 4*g + r%4, so the two lanes l and l ^ 32 hold all K scores of one
// point between them.  `ys` is y[K][P] in LDS.  Lanes whose point does not exist must not call this.
// unseen_zero: a point whose similarities are all exactly zero (the fused row of a point that no view sees is all
// zero) gets zero properties instead of what Eq. 4 gives for equal similarities, the mean of y.
template <int MT>
__device__ __forceinline__ void finish_scores(const scores_f32x16 (&acc)[MT], long long n, int g, int K, int P, float inv_T,
                                              const float* __restrict__ ys, float* __restrict__ scores,
                                              float* __restrict__ prop, int* __restrict__ label, bool unseen_zero = false) {
  float* __restrict__ srow = scores + n * K;
  const bool vec_store = (K & 3) == 0 && ((reinterpret_cast<uintptr_t>(scores) & 15) == 0);
  float best = -INFINITY;
  int bidx = 0;
  bool any_nonzero = false;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int m0 = mt * kScoreTileM + 8 * q + 4 * g;
      if (vec_store) {
        if (m0 < K) {
          scores_f32x4 v = {acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]};
          *reinterpret_cast<scores_f32x4*>(srow + m0) = v;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (m0 + e < K) srow[m0 + e] = acc[mt][4 * q + e];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float sc = acc[mt][4 * q + e];
        if (m0 + e < K && sc > best) { best = sc; bidx = m0 + e; }   // ascending m: lowest index wins ties
        any_nonzero = any_nonzero || (m0 + e < K && sc != 0.0f);
      }
    }
  {
    const float ob = __shfl_xor(best, 32, kWave);
    const int oi = __shfl_xor(bidx, 32, kWave);
    if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
  }
  if (label && g == 0) label[n] = bidx;
  if (!prop) return;
  const bool zero_row = unseen_zero && !(any_nonzero || __shfl_xor((int)any_nonzero, 32, kWave) != 0);

  float den = 0.0f, num[kScoreMaxP];
#pragma unroll
  for (int p = 0; p < kScoreMaxP; ++p) num[p] = 0.0f;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = mt * kScoreTileM + 8 * (r / 4) + 4 * g + (r & 3);
      if (m < K) {
        const float e = expf((acc[mt][r] - best) * inv_T);
        den += e;
#pragma unroll
        for (int p = 0; p < kScoreMaxP; ++p)
          if (p < P) num[p] = __builtin_fmaf(e, ys[m * P + p], num[p]);
      }
    }
  den += __shfl_xor(den, 32, kWave);
#pragma unroll
  for (int p = 0; p < kScoreMaxP; ++p) {
    if (p < P) {
      const float t = num[p] + __shfl_xor(num[p], 32, kWave);
      if (g == 0) prop[n * P + p] = zero_row ? 0.0f : t / den;
    }
  }
}

}  // namespace aura
