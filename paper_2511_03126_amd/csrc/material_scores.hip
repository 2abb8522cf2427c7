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
#include <algorithm>

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

// The same contraction for whole macro steps and 16-byte aligned rows, software-pipelined: what step s + 1 needs - the
// lane's 64 bytes of each of its RT rows and, with PRE_A, the split embeddings of the step (MT * 4 KiB, L2 hits) - is
// requested before the products of step s and kept in a second set of registers (the loop is unrolled by two, so
// that nothing that is still on its way has to be copied).  The memory counter returns reads in order: the requests
// for the next step are always the youngest, so waiting for this step's operands never waits for them.  Without the
// pipeline a wave asked for a step only when it needed it, and the kernel reached 4.0 of the 5.3 TB/s that the same
// read pattern reaches without arithmetic.  RT tiles of 32 points per wave share the embeddings of a step.
template <int MT, int RT, bool PRE_A>
__global__ __launch_bounds__(256) void k_material_scores_rt(ScoreArgs a) {
  __shared__ float ys[kMaxK * kMaxP];
  __shared__ __attribute__((aligned(16))) float s_stage[4][score_stage_floats<16>()];
  if (a.prop) {
    for (int t = threadIdx.x; t < a.K * a.P; t += blockDim.x) ys[t] = a.y[t];
  }
  __syncthreads();

  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const long long n0 = ((long long)blockIdx.x * 4 + wave) * (kTileN * RT);
  if (n0 >= a.N) return;
  const int g = lane / 32;
  const float* __restrict__ row[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const long long n = n0 + t * kTileN + (lane & 31);
    row[t] = a.fused + (n < a.N ? n : a.N - 1) * a.D + g * 16;
  }
  f32x16 acc[RT][MT];
#pragma unroll
  for (int t = 0; t < RT; ++t)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][mt][r] = 0.0f;

  struct Rows { f32x4 v[RT][4]; };
  struct Emb { bf16x8 hi[MT][2], lo[MT][2]; };
  auto load_rows = [&](int s, Rows& r) {
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) r.v[t][q] = *reinterpret_cast<const f32x4*>(row[t] + s * kStepK + 4 * q);
  };
  auto load_emb = [&](int s, Emb& e) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const bf16x8* slot = a.a_split + ((long long)(s * MT + mt) * 2 + j) * 2 * kWave + lane;
        e.hi[mt][j] = slot[0];
        e.lo[mt][j] = slot[kWave];
      }
  };
  auto products = [&](const Rows& r, const Emb& e) {
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      bf16x8 bh[2], bl[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const float x = r.v[t][2 * j + (c >> 2)][c & 3];
          const __bf16 h = (__bf16)x;
          bh[j][c] = h;
          bl[j][c] = (__bf16)(x - (float)h);
        }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[t][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(e.hi[mt][j], bh[j], acc[t][mt], 0, 0, 0);
          acc[t][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(e.hi[mt][j], bl[j], acc[t][mt], 0, 0, 0);
          acc[t][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(e.lo[mt][j], bh[j], acc[t][mt], 0, 0, 0);
        }
    }
  };

  const int last = a.steps - 1;
  Rows r0, r1;
  Emb e0, e1;
  load_rows(0, r0);
  if constexpr (PRE_A) load_emb(0, e0);
  for (int s = 0; s < a.steps; s += 2) {
    // step s from set 0 while step s + 1 arrives in set 1 (past the end: the last step again, read and not used)
    if constexpr (PRE_A) load_emb(min(s + 1, last), e1); else load_emb(s, e0);
    load_rows(min(s + 1, last), r1);
    __builtin_amdgcn_sched_barrier(0);
    products(r0, e0);
    __builtin_amdgcn_sched_barrier(0);
    if (s + 1 < a.steps) {   // uniform
      if constexpr (PRE_A) load_emb(min(s + 2, last), e0); else load_emb(s + 1, e1);
      load_rows(min(s + 2, last), r0);
      __builtin_amdgcn_sched_barrier(0);
      products(r1, e1);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const long long first = n0 + t * kTileN;
    const int rows = (int)std::min<long long>(kTileN, std::max<long long>(a.N - first, 0));
    finish_scores_staged<MT, 16>(acc[t], first, rows, lane, a.K, a.P, a.inv_T, ys, a.scores, a.prop, a.label,
                                 a.unseen_zero != 0, s_stage[wave]);
  }
}

// Where all the split embeddings of a call fit into LDS (steps * MT <= kLdsSlots blocks of 4 KiB: up to 1024 channels
// for 32 materials, 512 for 64), one workgroup of 16 waves per compute unit copies them there once and then walks over
// tiles of 32 points: the embeddings no longer come from L2 once per tile - reading them there costs the row stream 15 %
// of its rate (a read-only probe of the same pattern: 5.3 TB/s alone, 4.5 TB/s with those reads beside it).  The rows are
// requested one macro step ahead, across tile boundaries, so the stream never pauses.
constexpr int kLdsSlots = 32;

// kLdsWaves waves per workgroup: 16 for up to 32 materials (128 registers per wave), 8 for up to 64.
template <int MT, int kLdsWaves>
__global__ __launch_bounds__(kLdsWaves* kWave) void k_material_scores_lds(ScoreArgs a) {
  __shared__ float ys[MT * kTileM * kMaxP];
  __shared__ __attribute__((aligned(16))) bf16x8 s_a[kLdsSlots * 2 * 2 * kWave];   // 128 KiB
  constexpr int kStageRows = kLdsWaves > 8 ? 8 : 16;
  __shared__ __attribute__((aligned(16))) float s_stage[kLdsWaves][score_stage_floats<kStageRows>()];
  if (a.prop) {
    for (int t = threadIdx.x; t < a.K * a.P; t += blockDim.x) ys[t] = a.y[t];
  }
  for (int t = threadIdx.x; t < a.steps * MT * 2 * 2 * kWave; t += blockDim.x) s_a[t] = a.a_split[t];
  __syncthreads();

  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int g = lane / 32;
  const long long n_tiles = (a.N + kTileN - 1) / kTileN;
  const long long stride = (long long)gridDim.x * kLdsWaves;
  long long tile = (long long)blockIdx.x * kLdsWaves + wave;
  if (tile >= n_tiles) return;
  auto row_of = [&](long long tl) {
    const long long n = tl * kTileN + (lane & 31);
    return a.fused + (n < a.N ? n : a.N - 1) * a.D + g * 16;
  };
  struct Rows { f32x4 v[4]; };
  auto load_rows = [&](const float* __restrict__ row, int s, Rows& r) {
#pragma unroll
    for (int q = 0; q < 4; ++q) r.v[q] = *reinterpret_cast<const f32x4*>(row + s * kStepK + 4 * q);
  };
  f32x16 acc[MT];
  auto products = [&](const Rows& r, int s) {
    bf16x8 bh[2], bl[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float x = r.v[2 * j + (c >> 2)][c & 3];
        const __bf16 h = (__bf16)x;
        bh[j][c] = h;
        bl[j][c] = (__bf16)(x - (float)h);
      }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const bf16x8* slot = s_a + ((s * MT + mt) * 2 + j) * 2 * kWave + lane;
        const bf16x8 ah = slot[0], al = slot[kWave];
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh[j], acc[mt], 0, 0, 0);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl[j], acc[mt], 0, 0, 0);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh[j], acc[mt], 0, 0, 0);
      }
  };

  const int last = a.steps - 1;
  const float* __restrict__ row = row_of(tile);
  Rows r0, r1;
  load_rows(row, 0, r0);
  while (true) {
    const long long next = tile + stride;
    const float* __restrict__ row_next = row_of(next < n_tiles ? next : tile);   // no further tile: this one again, unused
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;
    for (int s = 0; s < a.steps; s += 2) {
      // step s from set 0 while step s + 1 arrives in set 1, and the other way round; after the tile's last step
      // the next tile's first
      if (s + 1 <= last) load_rows(row, s + 1, r1); else load_rows(row_next, 0, r1);
      __builtin_amdgcn_sched_barrier(0);
      products(r0, s);
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 <= last) {   // uniform
        if (s + 2 <= last) load_rows(row, s + 2, r0); else load_rows(row_next, 0, r0);
        __builtin_amdgcn_sched_barrier(0);
        products(r1, s + 1);
        __builtin_amdgcn_sched_barrier(0);
      } else {
        r0 = r1;   // odd number of steps: the next tile's first step sits in set 1
      }
    }
    finish_scores_staged<MT, kStageRows>(acc, tile * kTileN, (int)std::min<long long>(kTileN, a.N - tile * kTileN), lane, a.K,
                                         a.P, a.inv_T, ys, a.scores, a.prop, a.label, a.unseen_zero != 0, s_stage[wave]);
    if (next >= n_tiles) break;
    tile = next;
    row = row_next;
  }
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

#ifndef AURA_SCORES_RT
#define AURA_SCORES_RT 1
#endif

template <int MT>
static hipError_t launch_mt(const ScoreArgs& a, bool aligned, hipStream_t stream) {
  // embeddings of the next step in registers where they are few (up to 64 materials)
  constexpr int RT = MT == 1 ? AURA_SCORES_RT : 1;
  constexpr bool PRE_A = MT <= 2;
  if constexpr (MT <= 2) {
    if (aligned && a.D % kStepK == 0 && a.steps * MT <= kLdsSlots) {
      constexpr int kWaves = MT == 1 ? 16 : 8;
      int dev = 0, cus = 256;
      if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      const long long n_tiles = (a.N + kTileN - 1) / kTileN;
      // worth it from about six tiles per wave: with fewer, the waves that get one tile more than the others set the
      // time (200 000 points are 1.5 tiles per wave), and every workgroup pays for its copy of the embeddings
      if (n_tiles >= 6ll * cus * kWaves) {
        hipLaunchKernelGGL((k_material_scores_lds<MT, kWaves>), dim3((unsigned)cus), dim3(kWaves * kWave), 0, stream, a);
        return hipGetLastError();
      }
    }
  }
  if (aligned && a.D % kStepK == 0) {
    const long long per_group = 4ll * kTileN * RT;
    hipLaunchKernelGGL((k_material_scores_rt<MT, RT, PRE_A>), dim3((unsigned)((a.N + per_group - 1) / per_group)), dim3(256),
                       0, stream, a);
    return hipGetLastError();
  }
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
