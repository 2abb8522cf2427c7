// The matrix-core contraction shared by the scoring kernels: one wave multiplies the fp32 rows of its 32
// points with up to MT * 32 fp32 row vectors ("embeddings": material text embeddings, or the features of
// source points) that a preparation kernel has split into two bf16 terms in operand order.
#pragma once

#include "aura_device.hpp"

namespace aura {

typedef __bf16 sc_bf16x8 __attribute__((ext_vector_type(8)));
typedef float sc_f32x4 __attribute__((ext_vector_type(4)));
typedef float sc_f32x16 __attribute__((ext_vector_type(16)));

constexpr int kScoreStepK = 32;   // channels per macro step: lane group g = lane / 32 owns 16 of them

// Channel held by (macro step s, half j, lane group g, element e): the same map is used for both
// operands, so any order works as long as it is this one on both sides.
__device__ __forceinline__ int score_chan_of(int s, int j, int g, int e) { return s * kScoreStepK + g * 16 + j * 8 + e; }

// acc[mt] += E_mt . row^T over all channels: embeddings on the M side, points on the N side, so that lane
// l = 32 g + n ends up with element r of tile mt = <embedding mt*32 + 8*(r/4) + 4*g + r%4, row of point n>.
// fp32 operands are split into two bf16 terms (x = hi + lo) and three partial products hi*hi + hi*lo +
// lo*hi are accumulated in fp32 (error of a product of unit vectors near 1e-6).
// a_split: [steps][MT][2 (j)][2 (hi, lo)][64 lanes] x 8 bf16.  Returns the sum of squares of the channels
// this lane read (half of the row: add the value of lane l ^ 32 for the whole row) when WANT_SS.
template <int MT, bool ROWS_ALIGNED, bool WANT_SS>
__device__ __forceinline__ float score_products(const float* __restrict__ row, int D, int steps,
                                                const sc_bf16x8* __restrict__ a_split, int lane,
                                                sc_f32x16 (&acc)[MT]) {
  const int g = lane / 32;
  float ss = 0.0f;
  for (int s = 0; s < steps; ++s) {
    const int c0 = s * kScoreStepK + g * 16;
    float b[16];
    if (ROWS_ALIGNED && c0 + 16 <= D) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        sc_f32x4 v = *reinterpret_cast<const sc_f32x4*>(row + c0 + 4 * q);
        b[4 * q] = v[0]; b[4 * q + 1] = v[1]; b[4 * q + 2] = v[2]; b[4 * q + 3] = v[3];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) b[e] = (c0 + e < D) ? row[c0 + e] : 0.0f;
    }
    if (WANT_SS) {
#pragma unroll
      for (int e = 0; e < 16; ++e) ss = __builtin_fmaf(b[e], b[e], ss);
    }
    sc_bf16x8 bh[2], bl[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = b[8 * j + e];
        __bf16 h = (__bf16)x;
        bh[j][e] = h;
        bl[j][e] = (__bf16)(x - (float)h);
      }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const sc_bf16x8* slot = a_split + ((long long)(s * MT + mt) * 2 + j) * 2 * kWave + lane;
        const sc_bf16x8 ah = slot[0], al = slot[kWave];
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh[j], acc[mt], 0, 0, 0);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl[j], acc[mt], 0, 0, 0);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh[j], acc[mt], 0, 0, 0);
      }
    }
  }
  return ss;
}

// Splits `emb` [n_rows][D] fp32 into the operand order above (rows beyond n_rows and channels beyond D are
// zero); `out` holds split_embeddings_bytes(D, MT) bytes.
size_t split_embeddings_bytes(int D, int MT);
hipError_t launch_split_embeddings(const float* emb, int n_rows, int D, int MT, void* out, hipStream_t stream);

}  // namespace aura
