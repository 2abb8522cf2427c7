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
        const float e = weight_exp((acc[mt][r] - best) * inv_T);
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

// The same for a whole wave whose 32 points are consecutive in memory (n0 .. n0 + rows - 1 exist), with the scores
// going through a small LDS buffer of the wave's own (kScoreStageFloats floats) so that they reach memory in long runs:
// in the accumulator layout a store instruction writes 32 bytes of each of 32 rows, and those partial-line writes cost
// the scoring kernels up to a fifth of their time (6.4 M points x 24 materials: 0.53 of 2.9 ms).  ROWS rows at a time
// (16, or 8 where LDS is short) are laid out as [row][material] in the buffer and copied out sixteen bytes per lane,
// eight neighbouring lanes per row.  All 64 lanes call this, also those whose point does not exist.
constexpr int kScoreStagePitch = 36;   // floats: rows start 4 banks apart
template <int ROWS>
constexpr int score_stage_floats() { return ROWS * kScoreStagePitch; }

template <int MT, int ROWS>
__device__ __forceinline__ void finish_scores_staged(const scores_f32x16 (&acc)[MT], long long n0, int rows, int lane, int K,
                                                     int P, float inv_T, const float* __restrict__ ys,
                                                     float* __restrict__ scores, float* __restrict__ prop,
                                                     int* __restrict__ label, bool unseen_zero, float* stage) {
  const int pt = lane & 31, g = lane >> 5;
  const bool valid = pt < rows;
  const long long n = n0 + (valid ? pt : 0);
  if ((K & 3) == 0 && ((reinterpret_cast<uintptr_t>(scores) & 15) == 0)) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int cols = min(kScoreTileM, K - mt * kScoreTileM);   // a multiple of 4
      if (cols <= 0) continue;                                    // uniform
      const int per_row = cols >> 2;
#pragma unroll
      for (int part = 0; part < 32 / ROWS; ++part) {
        if (pt / ROWS == part) {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            *reinterpret_cast<scores_f32x4*>(stage + (pt % ROWS) * kScoreStagePitch + 8 * q + 4 * g) =
                scores_f32x4{acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]};
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (int idx = lane; idx < ROWS * per_row; idx += kWave) {
          const int r = idx / per_row, c4 = idx - r * per_row;
          const int row = part * ROWS + r;
          if (row < rows)
            *reinterpret_cast<scores_f32x4*>(scores + (n0 + row) * K + mt * kScoreTileM + 4 * c4) =
                *reinterpret_cast<const scores_f32x4*>(stage + r * kScoreStagePitch + 4 * c4);
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
  } else if (valid) {
    float* __restrict__ srow = scores + n * K;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * kScoreTileM + 8 * (r >> 2) + 4 * g + (r & 3);
        if (m < K) srow[m] = acc[mt][r];
      }
  }
  // label and Eq. 4 as in finish_scores; the two lanes of a point exchange with each other only
  float best = -INFINITY;
  int bidx = 0;
  bool any_nonzero = false;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {   // ascending material index within the lane: the lowest index wins ties
      const int m = mt * kScoreTileM + 8 * (r >> 2) + 4 * g + (r & 3);
      const float sc = acc[mt][r];
      if (m < K && sc > best) { best = sc; bidx = m; }
      any_nonzero = any_nonzero || (m < K && sc != 0.0f);
    }
  {
    const float ob = __shfl_xor(best, 32, kWave);
    const int oi = __shfl_xor(bidx, 32, kWave);
    if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
  }
  if (label && g == 0 && valid) label[n] = bidx;
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
        const float e = weight_exp((acc[mt][r] - best) * inv_T);
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
      if (g == 0 && valid) prop[n * P + p] = zero_row ? 0.0f : t / den;
    }
  }
}

// What finish_scores_staged writes for 32 consecutive points whose similarities are all exactly +0 (a tile that no view
// sees), without its exponentials: scores 0, label 0, and the properties Eq. 4 gives for equal similarities - the same
// sums in the same order (every weight is exp(0 * inv_T) = 1, so a fused multiply-add by it is an addition), hence the
// same bits - or zeros with unseen_zero.  All 64 lanes call this; the caller has checked that 0 * inv_T is 0.
template <int MT>
__device__ __forceinline__ void finish_zero_rows(long long n0, int rows, int lane, int K, int P, const float* __restrict__ ys,
                                                 float* __restrict__ scores, float* __restrict__ prop, int* __restrict__ label,
                                                 bool unseen_zero) {
  const int pt = lane & 31, g = lane >> 5;
  float* __restrict__ base = scores + n0 * K;
  const long long total = (long long)rows * K;
  if ((K & 3) == 0 && ((reinterpret_cast<uintptr_t>(base) & 15) == 0)) {
    for (long long i = 4 * lane; i < total; i += 4 * kWave) *reinterpret_cast<scores_f32x4*>(base + i) = scores_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  } else {
    for (long long i = lane; i < total; i += kWave) base[i] = 0.0f;
  }
  if (label && g == 0 && pt < rows) label[n0 + pt] = 0;
  if (!prop) return;
  float den = 0.0f, num[kScoreMaxP];
#pragma unroll
  for (int p = 0; p < kScoreMaxP; ++p) num[p] = 0.0f;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = mt * kScoreTileM + 8 * (r / 4) + 4 * g + (r & 3);
      if (m < K) {
        den += 1.0f;
#pragma unroll
        for (int p = 0; p < kScoreMaxP; ++p)
          if (p < P) num[p] = __builtin_fmaf(1.0f, ys[m * P + p], num[p]);
      }
    }
  den += __shfl_xor(den, 32, kWave);
#pragma unroll
  for (int p = 0; p < kScoreMaxP; ++p) {
    if (p < P) {
      const float t = num[p] + __shfl_xor(num[p], 32, kWave);
      if (g == 0 && pt < rows) prop[(n0 + pt) * P + p] = unseen_zero ? 0.0f : t / den;
    }
  }
}

}  // namespace aura
