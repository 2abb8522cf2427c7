// aura_knn_densify: Sec. 3.4.1 Eq. 5 - material vectors of dense query points from their k nearest
// source points in feature space (cosine similarity of the fused features), similarity-weighted mean,
// then the kernel regression of Eq. 4 on the interpolated vector.
//
// The similarities of all queries to all sources are one dense contraction [Ns x D] . [D x Nq], done on
// the matrix cores exactly like the material scores (sources on the M side, points on the N side, fp32
// operands as two bf16 terms, three partial products): a lane ends up with half the similarities of ONE
// query, lane l ^ 32 with the other half.  The selection of the k largest is k rounds of "largest value
// left" over the lane's registers plus one exchange with the partner lane (of equal values the lower
// source index first); both lanes of a pair keep the same list.  The weighted mean of the neighbours'
// vectors is evaluated directly in the accumulator layout of the scoring epilogue, which then stores it
// and applies Eq. 4.
//
// Like the scoring kernel this one is bound by reading the query features once from HBM.
#include "aura_device.hpp"
#include "launch.hpp"
#include "scores_core.hpp"
#include "scores_epilogue.hpp"

namespace aura {

constexpr int kKnnMaxK = 16;       // neighbours per query
constexpr int kKnnMaxSources = 256;

struct KnnArgs {
  const float* fq;          // [Nq][D]
  long long Nq;
  int D, Ns, K, P, k;
  const sc_bf16x8* a_split; // split source features
  int steps;
  const float* s_inv_norm;  // [Ns] 1 / |F(r_j)| (0 for a zero vector)
  const float* ws;          // [Ns][K]
  const float* y;
  float inv_T;
  float* wq;                // [Nq][K]
  float* prop;
  int* label;
  int* nn_idx;              // [Nq][k] or nullptr
};

__global__ __launch_bounds__(256) void k_source_norms(const float* __restrict__ fs, int Ns, int D, float* __restrict__ out) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int j = blockIdx.x * 4 + wave;
  if (j >= Ns) return;
  float ss = 0.0f;
  for (int c = lane; c < D; c += kWave) ss = __builtin_fmaf(fs[(long long)j * D + c], fs[(long long)j * D + c], ss);
  ss = wave_sum(ss);
  if (lane == 0) out[j] = ss > 0.0f ? 1.0f / sqrtf(ss) : 0.0f;
}

// The contraction of scores_core.hpp with the split source features of one macro step staged in LDS for the
// whole workgroup (double buffered, one barrier per step).  With several tiles of sources the operand block
// of a step is MT * 4 KiB and every wave needs all of it: read straight from L2 by every wave it is the
// bound of the kernel (Ns = 150: 590 KB per wave against 98 KB of query rows).  The next step's operand
// block and row channels are requested before this step's products.  Needs D to be a multiple of 32 and
// 16-byte aligned rows (no partial step); all 256 threads of the workgroup must call this together.
template <int MT>
__device__ __forceinline__ float score_products_staged(const float* __restrict__ row, int steps,
                                                       const sc_bf16x8* __restrict__ a_split, int lane,
                                                       sc_bf16x8* s_a, sc_f32x16 (&acc)[MT]) {
  constexpr int kBlock = MT * 2 * 2 * kWave;         // 16-byte operand slots per macro step = 256 * MT
  const int g = lane / 32;
  const float* __restrict__ mine = row + g * 16;     // the lane's 16 channels of step s: mine + 32 s
  float ss = 0.0f;
  sc_bf16x8 stage[MT];
  // The query rows are the stream from far memory, and with two waves per SIMD a compute unit has few of them in
  // flight: the channels of step s + 2 are requested at the start of step s, into the third of three register sets that
  // take turns (the loop is unrolled by three so that no set is copied while its reads are still on their way).
  sc_f32x4 r0[4], r1[4], r2[4];
  const int last = steps - 1;
  auto fetch = [&](int s, sc_f32x4 (&r)[4]) {
    const int sc = min(s, last);   // past the end: the last step again (read, not used)
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = *reinterpret_cast<const sc_f32x4*>(mine + 32 * sc + 4 * q);
  };
#pragma unroll
  for (int u = 0; u < MT; ++u) s_a[threadIdx.x + 256 * u] = a_split[threadIdx.x + 256 * u];
  fetch(0, r0);
  fetch(1, r1);
  __syncthreads();
  auto step = [&](int s, const sc_f32x4 (&b)[4], sc_f32x4 (&ahead)[4]) {
    const sc_bf16x8* cur = s_a + (s & 1) * kBlock;
    sc_bf16x8* nxt = s_a + ((s + 1) & 1) * kBlock;
    const int sn = min(s + 1, last);
#pragma unroll
    for (int u = 0; u < MT; ++u) stage[u] = a_split[(long long)sn * kBlock + threadIdx.x + 256 * u];
    fetch(s + 2, ahead);
    __builtin_amdgcn_sched_barrier(0);
    sc_bf16x8 bh[2], bl[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = b[2 * j + (e >> 2)][e & 3];
        ss = __builtin_fmaf(x, x, ss);
        const __bf16 h = (__bf16)x;
        bh[j][e] = h;
        bl[j][e] = (__bf16)(x - (float)h);
      }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const sc_bf16x8* slot = cur + (mt * 2 + j) * 2 * kWave + lane;
        const sc_bf16x8 ah = slot[0], al = slot[kWave];
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh[j], acc[mt], 0, 0, 0);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl[j], acc[mt], 0, 0, 0);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh[j], acc[mt], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < MT; ++u) nxt[threadIdx.x + 256 * u] = stage[u];
    __syncthreads();   // the next step's operands are in place; everybody is done with this step's
  };
  for (int s = 0; s < steps; s += 3) {   // `steps` is uniform over the workgroup: every wave passes the same barriers
    step(s, r0, r2);
    if (s + 1 < steps) step(s + 1, r1, r0);
    if (s + 2 < steps) step(s + 2, r2, r1);
  }
  return ss;
}

// MT: tiles of 32 sources; MTK: tiles of 32 materials.
template <int MT, int MTK, bool ROWS_ALIGNED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_knn_densify(KnnArgs a) {
  __shared__ float ys[kScoreMaxK * kScoreMaxP];
  __shared__ int s_idx[128 * kKnnMaxK];     // [point of the workgroup][round]: the neighbour list
  __shared__ float s_phi[128 * kKnnMaxK];
  __shared__ sc_bf16x8 s_a[ROWS_ALIGNED ? 2 * MT * 2 * 2 * kWave : 1];   // split source features of two macro steps
  if (a.prop) {
    for (int t = threadIdx.x; t < a.K * a.P; t += blockDim.x) ys[t] = a.y[t];
  }
  __syncthreads();

  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const long long n0 = ((long long)blockIdx.x * 4 + wave) * 32;   // a wave past the end still takes part in the staging
  const int g = lane / 32;
  const long long n = n0 + (lane & 31);
  const bool valid = n < a.Nq;
  const float* __restrict__ row = a.fq + (valid ? n : a.Nq - 1) * a.D;

  sc_f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;
  float ss;
  if constexpr (ROWS_ALIGNED)   // whole macro steps, 16-byte aligned rows: operands staged in LDS
    ss = score_products_staged<MT>(row, a.steps, a.a_split, lane, s_a, acc);
  else
    ss = score_products<MT, false, true>(row, a.D, a.steps, a.a_split, lane, acc);
  ss += __shfl_xor(ss, 32, kWave);
  const float q_inv = ss > 0.0f ? 1.0f / sqrtf(ss) : 0.0f;

  // cosine similarities; slots beyond Ns can never be selected
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
      acc[mt][r] = j < a.Ns ? acc[mt][r] * q_inv * a.s_inv_norm[j] : -INFINITY;
    }

  // ---- the k nearest sources, in order.  Both lanes of a pair find the same winner each round; the list goes
  // to LDS (one slot per point and round) so that the rounds can be a real loop without register arrays.
  const int ke = min(a.k, a.Ns);
  const int slot = (wave * 32 + (lane & 31)) * kKnnMaxK;
  float den = 0.0f;
#pragma unroll 1
  for (int t = 0; t < ke; ++t) {
    float best = -INFINITY;
    int bj = 0x7fffffff;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {   // ascending source index within the lane: the first of equal values stays
        const int j = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (acc[mt][r] > best) { best = acc[mt][r]; bj = j; }
      }
    const float ob = __shfl_xor(best, 32, kWave);
    const int oj = __shfl_xor(bj, 32, kWave);
    if (ob > best || (ob == best && oj < bj)) { best = ob; bj = oj; }
    if (g == 0) {
      s_idx[slot + t] = bj;
      s_phi[slot + t] = best;
    }
    den += best;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (j == bj) acc[mt][r] = -INFINITY;
      }
  }
  if (!valid) return;   // below: only LDS slots of the lane's own pair (written above by this wave) and lane ^ 32
  if (a.nn_idx && g == 0) {
    for (int t = 0; t < a.k; ++t) a.nn_idx[n * a.k + t] = t < ke ? s_idx[slot + t] : -1;
  }

  // ---- Eq. 5 in the layout of the scoring epilogue: element r of tile mt is material mt*32 + 8*(r/4) + 4*g + r%4
  const bool degenerate = fabsf(den) < 1e-12f;   // no usable weights: the nearest source's vector
  const float inv_den = degenerate ? 1.0f : 1.0f / den;
  sc_f32x16 out[MTK];
#pragma unroll
  for (int mt = 0; mt < MTK; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) out[mt][r] = 0.0f;
  const int n_used = degenerate ? 1 : ke;
#pragma unroll 1
  for (int t = 0; t < n_used; ++t) {
    const float w = degenerate ? 1.0f : s_phi[slot + t];
    const float* __restrict__ src = a.ws + (long long)s_idx[slot + t] * a.K;
#pragma unroll
    for (int mt = 0; mt < MTK; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (m < a.K) out[mt][r] = __builtin_fmaf(w, src[m], out[mt][r]);
      }
  }
#pragma unroll
  for (int mt = 0; mt < MTK; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) out[mt][r] *= inv_den;
  finish_scores<MTK>(out, n, g, a.K, a.P, a.inv_T, ys, a.wq, a.prop, a.label);
}

// ------------------------------------------------------------------------------------ host

static size_t knn_round256(size_t x) { return (x + 255) & ~(size_t)255; }
static int knn_source_tiles(int Ns) {
  const int mt = (Ns + 31) / 32;
  return mt <= 6 ? mt : 8;
}

bool knn_supported(int Ns, int K, int k, int P) {
  return Ns >= 1 && Ns <= kKnnMaxSources && K >= 1 && K <= kScoreMaxK && k >= 1 && k <= kKnnMaxK && P >= 0 && P <= kScoreMaxP;
}

size_t knn_workspace_bytes(int D, int Ns) {
  return knn_round256(split_embeddings_bytes(D, knn_source_tiles(Ns))) + knn_round256((size_t)Ns * sizeof(float));
}

template <int MT, int MTK>
static hipError_t launch_knn(const KnnArgs& a, bool aligned, hipStream_t stream) {
  const dim3 grid((unsigned)((a.Nq + 127) / 128)), block(256);
  if (aligned)
    hipLaunchKernelGGL((k_knn_densify<MT, MTK, true>), grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL((k_knn_densify<MT, MTK, false>), grid, block, 0, stream, a);
  return hipGetLastError();
}

template <int MT>
static hipError_t launch_knn_mtk(const KnnArgs& a, bool aligned, hipStream_t stream) {
  const int mtk = (a.K + 31) / 32;
  if (mtk <= 1) return launch_knn<MT, 1>(a, aligned, stream);
  if (mtk == 2) return launch_knn<MT, 2>(a, aligned, stream);
  return launch_knn<MT, 4>(a, aligned, stream);
}

hipError_t launch_knn_densify(const float* fq, long long Nq, int D, const float* fs, int Ns, const float* ws, int K,
                              int k, const float* y, int P, float temperature, float* wq, float* prop, int* label,
                              int* nn_idx, void* workspace, hipStream_t stream) {
  if (Nq == 0) return hipSuccess;
  const int MT = knn_source_tiles(Ns);
  char* base = static_cast<char*>(workspace);
  void* split = base;
  float* inv_norm = reinterpret_cast<float*>(base + knn_round256(split_embeddings_bytes(D, MT)));
  hipError_t e = launch_split_embeddings(fs, Ns, D, MT, split, stream);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_source_norms, dim3((unsigned)((Ns + 3) / 4)), dim3(256), 0, stream, fs, Ns, D, inv_norm);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  KnnArgs a{fq, Nq, D, Ns, K, P, k, static_cast<const sc_bf16x8*>(split), (D + kScoreStepK - 1) / kScoreStepK, inv_norm, ws,
            y, 1.0f / temperature, wq, prop, label, nn_idx};
  const bool aligned = (D & 31) == 0 && (reinterpret_cast<uintptr_t>(fq) & 15) == 0;
  switch (MT) {
    case 1: return launch_knn_mtk<1>(a, aligned, stream);
    case 2: return launch_knn_mtk<2>(a, aligned, stream);
    case 3: return launch_knn_mtk<3>(a, aligned, stream);
    case 4: return launch_knn_mtk<4>(a, aligned, stream);
    case 5: return launch_knn_mtk<5>(a, aligned, stream);
    case 6: return launch_knn_mtk<6>(a, aligned, stream);
    default: return launch_knn_mtk<8>(a, aligned, stream);
  }
}

}  // namespace aura
