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
// The source features are divided by their norms before they are split into operand order, so the
// accumulators are <q, s / |s|>: the order of a query's similarities does not depend on its own norm, which
// only scales the weights at the end.
//
// A workgroup is eight waves (256 queries) that share the split source features of a channel step through
// LDS: the block is as large as the query rows of 160 queries, so the fewer workgroups fetch it the better.
#include "aura_device.hpp"
#include "launch.hpp"
#include "scores_core.hpp"
#include "scores_epilogue.hpp"

namespace aura {

constexpr int kKnnMaxK = 16;       // neighbours per query
constexpr int kKnnMaxSources = 256;
// Waves per workgroup.  The waves of a workgroup share the operand blocks and move in step with each other through the
// barrier of every channel step: they select, and leave the memory system idle, at the same time.  Up to 160 sources
// (blocks of 20 KB) two workgroups of four waves fit a compute unit and drift apart (200 000 queries, 150 sources: 0.270
// against 0.287 ms with one workgroup of eight); beyond that one workgroup of eight, which fetches every block once.
constexpr int knn_waves(int MT) { return MT <= 5 ? 4 : 8; }
constexpr int kKnnLdsVectors = 6144;    // floats of LDS for the sources' material vectors [Ns][K]; larger sets are read from memory

struct KnnArgs {
  const float* fq;          // [Nq][D]
  long long Nq;
  int D, Ns, K, P, k;
  const sc_bf16x8* a_split; // split source features
  int steps;
  const float* ws;          // [Ns][K]
  const float* y;
  float inv_T;
  float* wq;                // [Nq][K]
  float* prop;
  int* label;
  int* nn_idx;              // [Nq][k] or nullptr
  long long n_tiles;        // tiles of 32 queries
  int n_ranges;             // contiguous ranges of tiles (see the kernel)
};

// The source features divided by their norms (a zero vector stays zero: similarity 0 to everything), split into
// two bf16 terms in the operand order of scores_core.hpp.  One wave per source slot (slots beyond Ns are zero): the
// wave adds up the squares of its source's channels, then every lane writes the 8-channel pieces (step, half, lane
// group) that the slot's operand lane holds.
__global__ __launch_bounds__(256) void k_split_sources(const float* __restrict__ fs, int Ns, int D, int MT, int steps,
                                                       __bf16* __restrict__ out) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int m = blockIdx.x * 4 + wave;
  if (m >= MT * 32) return;
  float scale = 0.0f;
  if (m < Ns) {   // uniform over the wave
    float ss = 0.0f;
    for (int c = lane; c < D; c += kWave) ss = __builtin_fmaf(fs[(long long)m * D + c], fs[(long long)m * D + c], ss);
    ss = wave_sum(ss);
    scale = ss > 0.0f ? 1.0f / sqrtf(ss) : 0.0f;
  }
  const int mt = m / 32;
  for (int piece = lane; piece < steps * 4; piece += kWave) {
    const int g = piece & 1, j = (piece >> 1) & 1, s = piece >> 2;
    __bf16* hi = out + ((((long long)(s * MT + mt) * 2 + j) * 2 + 0) * kWave + g * 32 + (m & 31)) * 8;
    __bf16* lo = hi + kWave * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = score_chan_of(s, j, g, e);
      const float x = (m < Ns && c < D) ? fs[(long long)m * D + c] * scale : 0.0f;
      const __bf16 h = (__bf16)x;
      hi[e] = h;
      lo[e] = (__bf16)(x - (float)h);
    }
  }
}

// The contraction of scores_core.hpp with the split source features of one macro step staged in LDS for the
// whole workgroup (double buffered, one barrier per step).  With several tiles of sources the operand block
// of a step is MT * 4 KiB and every wave needs all of it: read straight from L2 by every wave it is the
// bound of the kernel (Ns = 150: 590 KB per wave against 98 KB of query rows).
//
// A wave's step is a chain - requests, conversion, LDS reads, products, LDS writes, barrier - and with two waves per
// SIMD, all in step with each other through the barrier, nothing hides one link behind another unless the wave does it
// itself.  So the step is laid out by hand (scheduling barriers keep the order): the operands of the next pair of
// (tile, half) groups are read from LDS while the matrix cores work on the current pair, whose two accumulators take
// turns so that no product waits for the one before it; the memory requests of the step (query channels three steps
// ahead, the operand block two steps ahead) are issued one at a time between the pairs, because eight waves that
// issue all of theirs at the same moment queue at the compute unit's one address unit; the operand block is written
// to LDS a full step after it was requested.
// Needs D to be a multiple of 32 and 16-byte aligned rows (no partial step); all threads of the workgroup must call
// this together; a wave without queries of its own (`work` false, uniform over the wave) only copies its share of the
// operand blocks and passes the barriers.
template <int MT>
__device__ __forceinline__ float score_products_staged(const float* __restrict__ row, int steps,
                                                       const sc_bf16x8* __restrict__ a_split, int lane,
                                                       sc_bf16x8* s_a, sc_f32x16 (&acc)[MT], bool work) {
  constexpr int kBlock = MT * 2 * 2 * kWave;         // 16-byte operand slots per macro step = 256 * MT
  constexpr int kKnnThreads = knn_waves(MT) * kWave;
  constexpr int kCopies = (kBlock + kKnnThreads - 1) / kKnnThreads;   // 16-byte slots a thread copies per step
  constexpr int kGroups = 2 * MT;                    // (half j, tile mt) groups of a step, j-major: three products each
  constexpr int kPairs = (kGroups + 1) / 2;          // neighbouring groups: different accumulators whenever MT > 1
  constexpr int kLoads = 4 + kCopies;                // memory requests of a step
  const int g = lane / 32;
  const float* __restrict__ mine = row + g * 16;     // the lane's 16 channels of step s: mine + 32 s
  float ss = 0.0f;
  sc_bf16x8 stage[kCopies];
  sc_f32x4 r0[4], r1[4], r2[4];
  const int last = steps - 1;                        // requests past the end take the last step again (read, not used)
  auto load_row = [&](int s, int q, sc_f32x4 (&r)[4]) {
    r[q] = *reinterpret_cast<const sc_f32x4*>(mine + 32 * min(s, last) + 4 * q);
  };
  auto load_block = [&](int s, int u) {
    if (threadIdx.x + kKnnThreads * u < kBlock)
      stage[u] = a_split[(long long)min(s, last) * kBlock + threadIdx.x + kKnnThreads * u];
  };
  // before the loop: block 0 in LDS, block 1 in the staging registers, the channels of steps 0 .. 2 on their way
#pragma unroll
  for (int u = 0; u < kCopies; ++u)
    if (threadIdx.x + kKnnThreads * u < kBlock) s_a[threadIdx.x + kKnnThreads * u] = a_split[threadIdx.x + kKnnThreads * u];
#pragma unroll
  for (int u = 0; u < kCopies; ++u) load_block(1, u);
  if (work) {
#pragma unroll
    for (int q = 0; q < 4; ++q) load_row(0, q, r0);
#pragma unroll
    for (int q = 0; q < 4; ++q) load_row(1, q, r1);
#pragma unroll
    for (int q = 0; q < 4; ++q) load_row(2, q, r2);
  }
  __syncthreads();
  // step s: `b` holds its channels and is free for the channels of step s + 3 once they are converted
  auto step = [&](int s, sc_f32x4 (&b)[4]) {
    const sc_bf16x8* cur = s_a + (s & 1) * kBlock;
    sc_bf16x8* nxt = s_a + ((s + 1) & 1) * kBlock;
    // the block of step s + 1, requested during step s - 1
#pragma unroll
    for (int u = 0; u < kCopies; ++u)
      if (threadIdx.x + kKnnThreads * u < kBlock) nxt[threadIdx.x + kKnnThreads * u] = stage[u];
    if (!work) {
#pragma unroll
      for (int u = 0; u < kCopies; ++u) load_block(s + 2, u);
      __syncthreads();
      return;
    }
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
    sc_bf16x8 ah[2][2], al[2][2];   // [register set][member of the pair]
    auto read_pair = [&](int p, int set) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int gi = 2 * p + i;
        if (gi < kGroups) {
          const sc_bf16x8* slot = cur + ((gi % MT) * 2 + gi / MT) * 2 * kWave + lane;
          ah[set][i] = slot[0];
          al[set][i] = slot[kWave];
        }
      }
    };
    read_pair(0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 0; p < kPairs; ++p) {
      const int set = p & 1;
      if (p + 1 < kPairs) read_pair(p + 1, set ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      const int g0 = 2 * p, g1 = 2 * p + 1;
      const int j0 = g0 / MT, m0 = g0 % MT, j1 = g1 / MT, m1 = g1 % MT;
      acc[m0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[set][0], bh[j0], acc[m0], 0, 0, 0);
      if (g1 < kGroups) acc[m1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[set][1], bh[j1], acc[m1], 0, 0, 0);
      acc[m0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[set][0], bl[j0], acc[m0], 0, 0, 0);
      if (g1 < kGroups) acc[m1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[set][1], bl[j1], acc[m1], 0, 0, 0);
      acc[m0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[set][0], bh[j0], acc[m0], 0, 0, 0);
      if (g1 < kGroups) acc[m1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[set][1], bh[j1], acc[m1], 0, 0, 0);
      // this pair's share of the step's memory requests: first the channels of step s + 3, then the block of step s + 2
#pragma unroll
      for (int k = p; k < kLoads; k += kPairs) {
        if (k < 4) load_row(s + 3, k, b);
        else load_block(s + 2, k - 4);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();   // the next step's operands are in place; everybody is done with this step's
  };
  for (int s = 0; s < steps; s += 3) {   // `steps` is uniform over the workgroup: every wave passes the same barriers
    step(s, r0);
    if (s + 1 < steps) step(s + 1, r1);
    if (s + 2 < steps) step(s + 2, r2);
  }
  return ss;
}

// MT: tiles of 32 sources; MTK: tiles of 32 materials.
template <int MT, int MTK, bool ROWS_ALIGNED>
__global__ __launch_bounds__(knn_waves(MT) * kWave) __attribute__((amdgpu_waves_per_eu(2))) void k_knn_densify(KnnArgs a) {
  constexpr int kKnnWaves = knn_waves(MT);
  __shared__ float ys[kScoreMaxK * kScoreMaxP];
  __shared__ float s_ws[kKnnLdsVectors];                // the sources' material vectors, when they fit
  __shared__ float s_out[kKnnWaves * score_stage_floats<16>()];   // per wave: score rows on their way to memory
  __shared__ sc_bf16x8 s_a[ROWS_ALIGNED ? 2 * MT * 2 * 2 * kWave : 1];   // split source features of two macro steps
  if (a.prop) {
    for (int t = threadIdx.x; t < a.K * a.P; t += blockDim.x) ys[t] = a.y[t];
  }
  const bool ws_in_lds = a.Ns * a.K <= kKnnLdsVectors;   // uniform
  if (ws_in_lds) {
    for (int t = threadIdx.x; t < a.Ns * a.K; t += blockDim.x) s_ws[t] = a.ws[t];
  }
  __syncthreads();

  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int g = lane / 32;
  const int ke = min(a.k, a.Ns);
  // The tiles are divided evenly into a.n_ranges contiguous ranges (one per compute unit), and workgroup b takes the
  // (b / n_ranges)-th eight tiles of range b % n_ranges: all workgroups but a range's last are full, and the ranges'
  // last workgroups, with few waves each, run side by side at the end, instead of a few full workgroups running
  // alone after all the others (200 000 queries are 3.05 rounds of full workgroups on 256 compute units).
  const int range = blockIdx.x % a.n_ranges;
  const long long t0 = a.n_tiles * range / a.n_ranges + (long long)(blockIdx.x / a.n_ranges) * kKnnWaves;
  const long long t_end = a.n_tiles * (range + 1) / a.n_ranges;
  if (t0 >= t_end) return;   // uniform over the workgroup, before its first barrier
  const long long tile = t0 + wave;
  const bool active = tile < t_end;                    // a wave without a tile still takes part in the staging
  const long long n0 = tile * 32;
  const long long n = n0 + (lane & 31);
  const bool valid = active && n < a.Nq;
  const float* __restrict__ row = a.fq + (valid ? n : a.Nq - 1) * a.D;

  sc_f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;
  float ss;
  if constexpr (ROWS_ALIGNED)   // whole macro steps, 16-byte aligned rows: operands staged in LDS
    ss = score_products_staged<MT>(row, a.steps, a.a_split, lane, s_a, acc, active);
  else
    ss = score_products<MT, false, true>(row, a.D, a.steps, a.a_split, lane, acc);
  ss += __shfl_xor(ss, 32, kWave);
  const float q_inv = ss > 0.0f ? 1.0f / sqrtf(ss) : 0.0f;

  // Slots beyond Ns can never be selected (they can only be in the last two tiles: MT = ceil(Ns / 32), or 8 for 7).
#pragma unroll
  for (int mt = (MT > 2 ? MT - 2 : 0); mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
      if (j >= a.Ns) acc[mt][r] = -INFINITY;
    }

  if (!active) return;   // no barrier below; only LDS of the wave's own (its part of s_out) and what was filled before the loop

  // ---- the k nearest sources, in order, and Eq. 5 along the way.  The accumulators are <q, s/|s|>, the cosine
  // similarities times |q|: the same order.  A round scans the lane's values in four independent chains (each in
  // ascending source index, so the first of equal values stays; a single chain is one long run of dependent
  // instructions), merges them, and exchanges with the partner lane; both lanes of a pair find the same winner.  The
  // winner's material vector is requested at once and added, weighted, after the round's marking pass.  Eq. 5 in the
  // layout of the scoring epilogue: element r of tile mt is material mt*32 + 8*(r/4) + 4*g + r%4; a material index
  // beyond K reads the last material instead, into an element that the epilogue never looks at.
  sc_f32x16 out[MTK];
#pragma unroll
  for (int mt = 0; mt < MTK; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) out[mt][r] = 0.0f;
  const int k_last = a.K - 1;
  float den = 0.0f;
  int nearest = 0;
#pragma unroll 1
  for (int t = 0; t < ke; ++t) {
    float cb[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    int cj[4] = {0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff};   // source index without the lane group's 4 g: a constant per element
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (acc[mt][r] > cb[r & 3]) { cb[r & 3] = acc[mt][r]; cj[r & 3] = mt * 32 + 8 * (r >> 2) + (r & 3); }
    auto merge = [](float& v, int& j, float ov, int oj) {   // larger value; of equal values the lower index
      if (ov > v || (ov == v && oj < j)) { v = ov; j = oj; }
    };
    merge(cb[0], cj[0], cb[1], cj[1]);
    merge(cb[2], cj[2], cb[3], cj[3]);
    merge(cb[0], cj[0], cb[2], cj[2]);
    float best = cb[0];
    int bj = cj[0] == 0x7fffffff ? cj[0] : cj[0] + 4 * g;
    merge(best, bj, __shfl_xor(best, 32, kWave), __shfl_xor(bj, 32, kWave));
    // Nothing compares greater when every similarity left is NaN (a NaN in the features): the round must still name
    // a source, because it addresses the sources' vectors.
    if ((unsigned)bj >= (unsigned)a.Ns) { bj = 0; best = 0.0f; }
    const float phi = best * q_inv;   // the cosine similarity
    den += phi;
    if (t == 0) nearest = bj;
    if (a.nn_idx && g == 0 && valid) a.nn_idx[n * a.k + t] = bj;
    // the first 32 materials' values are requested before the marking pass and used after it
    int kl = k_last;
    asm volatile("" : "+v"(kl));   // the clamped material indices are recomputed every round instead of living in 16 registers per tile
    auto read_vector = [&](int mt, float (&v)[16]) {
      if (ws_in_lds) {   // uniform.  (Two branches, so that the reads of the LDS copy are LDS instructions and not generic ones.)
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = s_ws[bj * a.K + min(mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3), kl)];
      } else {
        const float* __restrict__ src = a.ws + (long long)bj * a.K;
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = src[min(mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3), kl)];
      }
    };
    float v0[16];
    read_vector(0, v0);
    const int bj_lane = bj - 4 * g;   // the winner's index as this lane's elements count
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (mt * 32 + 8 * (r >> 2) + (r & 3) == bj_lane) acc[mt][r] = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) out[0][r] = __builtin_fmaf(phi, v0[r], out[0][r]);
#pragma unroll
    for (int mt = 1; mt < MTK; ++mt) {
      float v[16];
      read_vector(mt, v);
#pragma unroll
      for (int r = 0; r < 16; ++r) out[mt][r] = __builtin_fmaf(phi, v[r], out[mt][r]);
    }
  }
  if (a.nn_idx && g == 0 && valid) {
    for (int t = ke; t < a.k; ++t) a.nn_idx[n * a.k + t] = -1;
  }
  if (fabsf(den) < 1e-12f) {   // no usable weights (a query without features, for one): the nearest source's vector
    if (ws_in_lds) {
#pragma unroll
      for (int mt = 0; mt < MTK; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[mt][r] = s_ws[nearest * a.K + min(mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3), k_last)];
    } else {
      const float* __restrict__ src = a.ws + (long long)nearest * a.K;
#pragma unroll
      for (int mt = 0; mt < MTK; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[mt][r] = src[min(mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3), k_last)];
    }
  } else {
    const float inv_den = 1.0f / den;
#pragma unroll
    for (int mt = 0; mt < MTK; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) out[mt][r] *= inv_den;
  }
  const int rows = (int)min((long long)32, a.Nq - n0);
  finish_scores_staged<MTK, 16>(out, n0, rows, lane, a.K, a.P, a.inv_T, ys, a.wq, a.prop, a.label, false,
                                s_out + wave * score_stage_floats<16>());
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
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  KnnArgs b = a;
  b.n_ranges = (int)(a.n_tiles < cus ? a.n_tiles : cus);
  const long long longest = (a.n_tiles + b.n_ranges - 1) / b.n_ranges;   // tiles of the longest range
  constexpr int kKnnWaves = knn_waves(MT);
  const dim3 grid((unsigned)(((longest + kKnnWaves - 1) / kKnnWaves) * b.n_ranges)), block(kKnnWaves * kWave);
  if (aligned)
    hipLaunchKernelGGL((k_knn_densify<MT, MTK, true>), grid, block, 0, stream, b);
  else
    hipLaunchKernelGGL((k_knn_densify<MT, MTK, false>), grid, block, 0, stream, b);
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
  const int steps = (D + kScoreStepK - 1) / kScoreStepK;
  hipLaunchKernelGGL(k_split_sources, dim3((unsigned)(MT * 32 / 4)), dim3(256), 0, stream, fs, Ns, D, MT, steps,
                     static_cast<__bf16*>(split));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  KnnArgs a{fq, Nq, D, Ns, K, P, k, static_cast<const sc_bf16x8*>(split), steps, ws,
            y, 1.0f / temperature, wq, prop, label, nn_idx, (Nq + 31) / 32, 1};
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
