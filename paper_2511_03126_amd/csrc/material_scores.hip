// aura_material_scores: Sec. 3.4.1 - similarity omega_k = <fused, temb_k> and the kernel
// regression of Eq. 4, plus the arg-max material label.
//
// The contraction [K x D] . [D x N] runs on the matrix cores (v_mfma_f32_32x32x16_bf16) with the
// materials on the M side and the points on the N side, so that one lane ends up holding half of
// the scores of ONE point: the softmax over materials is then an in-register reduction plus a
// single exchange between lane l and lane l ^ 32.  fp32 operands are split into two bf16 terms
// (x = hi + lo) and three partial products hi*hi + hi*lo + lo*hi are accumulated in fp32, which
// keeps the error of a score of unit vectors near 1e-6.
//
// The kernel is bound by reading fused[N][D] once from HBM (arithmetic intensity 2K/(4+4K/D)
// flop per byte, far below the machine balance): the matrix cores are the right instruction,
// not the bound.  The text embeddings are split once per call by a small preparation kernel into
// the workspace, already in the per-lane operand order, and stay resident in L2.
#include "aura_device.hpp"
#include "launch.hpp"
#include "scores_core.hpp"
#include "scores_epilogue.hpp"

namespace aura {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTileM = 32;      // materials per MFMA tile
constexpr int kTileN = 32;      // points per wave
constexpr int kStepK = 32;      // channels per macro step: lane group g = lane / 32 owns 16 of them
constexpr int kMaxP = 8;
constexpr int kMaxK = 128;

struct ScoreArgs {
  const float* fused;
  long long N;
  int D, K, P;
  const float* y;
  float inv_T;
  int unseen_zero;
  float* scores;
  float* prop;
  int* label;
  const bf16x8* a_split;   // workspace: [S][MT][2 (j)][2 (hi, lo)][64 lanes] x 8 bf16
  int steps;               // S = ceil(D / 32)
};

__global__ __launch_bounds__(256) void k_split_embeddings(const float* __restrict__ temb, int K, int D, int MT,
                                                          int steps, __bf16* __restrict__ out) {
  long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;   // one thread per (slot, lane)
  long long total = (long long)steps * MT * 2 * kWave;
  if (t >= total) return;
  int lane = t % kWave;
  int j = (t / kWave) % 2;
  int mt = (t / (kWave * 2)) % MT;
  int s = t / ((long long)kWave * 2 * MT);
  int m = mt * kTileM + lane % 32, g = lane / 32;
  __bf16* hi = out + ((((long long)(s * MT + mt) * 2 + j) * 2 + 0) * kWave + lane) * 8;
  __bf16* lo = out + ((((long long)(s * MT + mt) * 2 + j) * 2 + 1) * kWave + lane) * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    int c = score_chan_of(s, j, g, e);
    float x = (m < K && c < D) ? temb[(long long)m * D + c] : 0.0f;
    __bf16 h = (__bf16)x;
    hi[e] = h;
    lo[e] = (__bf16)(x - (float)h);
  }
}

template <int MT, bool ROWS_ALIGNED>
__global__ __launch_bounds__(256) void k_material_scores(ScoreArgs a) {
  __shared__ float ys[kMaxK * kMaxP];
  if (a.prop) {
    for (int t = threadIdx.x; t < a.K * a.P; t += blockDim.x) ys[t] = a.y[t];
  }
  __syncthreads();

  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const long long n0 = ((long long)blockIdx.x * 4 + wave) * kTileN;
  if (n0 >= a.N) return;
  const int g = lane / 32;
  const long long n = n0 + (lane & 31);
  const bool valid = n < a.N;
  const float* __restrict__ row = a.fused + (valid ? n : a.N - 1) * a.D;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;

  score_products<MT, ROWS_ALIGNED, false>(row, a.D, a.steps, a.a_split, lane, acc);

  if (!valid) return;   // no cross-lane traffic below except with lane ^ 32, which holds the same point
  finish_scores<MT>(acc, n, g, a.K, a.P, a.inv_T, ys, a.scores, a.prop, a.label, a.unseen_zero != 0);
}

size_t split_embeddings_bytes(int D, int MT) {
  return (size_t)((D + kStepK - 1) / kStepK) * MT * 2 * 2 * kWave * 8 * sizeof(__bf16);
}

hipError_t launch_split_embeddings(const float* emb, int n_rows, int D, int MT, void* out, hipStream_t stream) {
  const int S = (D + kStepK - 1) / kStepK;
  const long long total = (long long)S * MT * 2 * kWave;
  hipLaunchKernelGGL(k_split_embeddings, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, emb, n_rows, D,
                     MT, S, static_cast<__bf16*>(out));
  return hipGetLastError();
}

static int tiles_m(int K) { return (K + kTileM - 1) / kTileM; }
static int steps_k(int D) { return (D + kStepK - 1) / kStepK; }

size_t scores_split_bytes(int D, int K) {
  int MT = tiles_m(K);
  if (MT == 3) MT = 4;
  return (size_t)steps_k(D) * MT * 2 * 2 * kWave * 8 * sizeof(__bf16);
}

// the split embeddings, then room for an fp32 copy of embeddings that arrive as 16-bit values
size_t scores_workspace_bytes(int D, int K) {
  return scores_split_bytes(D, K) + (((size_t)K * D * sizeof(float) + 255) & ~(size_t)255);
}

// Text embeddings given as bf16 (dtype 1) or fp16 (dtype 2) values, widened exactly to fp32.
__global__ __launch_bounds__(256) void k_widen_embeddings(const uint16_t* __restrict__ src, int dtype, long long n,
                                                          float* __restrict__ dst) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint16_t b = src[i];
  dst[i] = dtype == 1 ? __uint_as_float((uint32_t)b << 16) : (float)__builtin_bit_cast(_Float16, b);
}

hipError_t launch_widen_embeddings(const void* src, int dtype, long long n, float* dst, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_widen_embeddings, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const uint16_t*>(src), dtype, n, dst);
  return hipGetLastError();
}

template <int MT>
static hipError_t launch_mt(const ScoreArgs& a, bool aligned, hipStream_t stream) {
  dim3 grid((unsigned)((a.N + 4 * kTileN - 1) / (4 * kTileN))), block(256);
  if (aligned)
    hipLaunchKernelGGL((k_material_scores<MT, true>), grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL((k_material_scores<MT, false>), grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_material_scores(const float* fused, long long N, int D, const float* temb, int K,
                                  const float* y, int P, float temperature, float* scores, float* prop,
                                  int* label, void* workspace, hipStream_t stream, int unseen_zero) {
  if (N == 0) return hipSuccess;
  int MT = tiles_m(K);
  if (MT == 3) MT = 4;
  const int S = steps_k(D);
  {
    long long total = (long long)S * MT * 2 * kWave;
    hipLaunchKernelGGL(k_split_embeddings, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, temb, K, D,
                       MT, S, static_cast<__bf16*>(workspace));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  ScoreArgs a{fused, N, D, K, P, y, 1.0f / temperature, unseen_zero, scores, prop, label,
              static_cast<const bf16x8*>(workspace), S};
  const bool aligned = (D & 3) == 0 && (reinterpret_cast<uintptr_t>(fused) & 15) == 0;
  switch (MT) {
    case 1: return launch_mt<1>(a, aligned, stream);
    case 2: return launch_mt<2>(a, aligned, stream);
    default: return launch_mt<4>(a, aligned, stream);
  }
}

}  // namespace aura
