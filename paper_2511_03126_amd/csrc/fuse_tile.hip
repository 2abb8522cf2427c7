// aura_fuse_features, matrix-core path (Sec. 3.1 "Feature Aggregation", Eq. 2).
//
// Eq. 2 with bilinear sampling is a weighted sum of feature cells:
//     sum_v M_vis(x_i, v) F_v(pi(x_i, v)) = sum_c  w[i][c] * F[c],
// where c runs over (view, cell) pairs and w[i][c] is the bilinear weight of cell c for point i
// (zero unless the view sees the point and c is one of the four cells around the projection).
// For a tile of 32 spatially neighbouring points only about a hundred cells carry a non-zero
// weight, so the sum is a small dense product
//     [32 points x L cells] . [L cells x D channels]
// that runs on the matrix cores with the stored 16-bit features as they are.  The gather
// formulation reads every cell row once per point and view (4 D elements per pair) and spends
// its time widening and multiplying on the vector ALUs; here each cell of the list is read once
// per tile.
//
// Two kernels:
//
// k_tile_prepare (one workgroup of 256 threads per tile, little register state, many tiles in
// flight per CU so that the projection -> depth-read -> list chain of one tile hides behind the
// others):
//   A  every (point, view) pair is projected and tested (Eq. 1, the shared fp32 decision
//      functions).  Per view, the bounding box of the touched cells is found with a half-wave
//      reduction.
//   B  views whose box fits 32 x 32 cells mark the touched cells in a 1024-bit map (exact list,
//      no duplicates, no untouched cells); larger boxes (points far apart) give each visible
//      pair four private entries.  A scan over the views lays the per-view lists end to end.
//   C  per chunk of the list: the weights are scattered into a [32][cells] matrix in LDS, split
//      into two 16-bit terms (hi + lo, about 16 mantissa bits), and copied out as k-steps of 16
//      cells in the operand layout of the matrix-core instruction.  Every tile owns a fixed number
//      of k-steps of storage; a tile that needs more (points far apart) is fused on the spot by a
//      plain gather, so which way a tile goes depends on the tile alone and results are
//      reproducible bit for bit.
//
// k_tile_product (one workgroup per tile, wave s owns channels [256 s, 256 s + 256)): per k-step
// each lane reads two 8-byte pieces (4 channels each, 128 channels apart) of 8 cell rows straight
// from global memory (the rows of a tile's neighbours keep them in L2), regroups them with byte
// permutes into the 8 B-operands and issues v_mfma_f32_32x32x16 with the hi and the lo weights.
// No barrier inside the loop; reads run two k-steps ahead of the products.  Then mean, L2 norm
// (half-wave reduction, across the waves through LDS) and streaming stores.
// Accumulator t = 4 h + j, register r of lane l is point 8 (r/4) + 4 (l/32) + r%4, channel
// 256 s + 128 h + 4 (l%32) + j: a store instruction writes 16 bytes per lane and the 32 lanes of
// a half wave cover 512 contiguous bytes of a row (full cache lines; writing 16 of every 32
// bytes, as a lane owning 8 consecutive channels would, halves the achieved write bandwidth).
//
// List entries that only pad the last k-step have zero weights, so feature maps must be finite.
#include <algorithm>

#include "aura_device.hpp"
#include "fuse_args.hpp"
#include "launch.hpp"
#include "scores_epilogue.hpp"
#include "timing.hpp"

namespace aura {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr int kViewBatch = 32;                 // views handled per pass over the point tile
constexpr int kPrepThreads = 256;
constexpr int kSlots = kPrepThreads / kTilePts;   // views processed side by side (one per half wave)
constexpr int kNIT = kViewBatch / kSlots;      // (point, view) pairs per thread and batch
#ifndef AURA_CHUNK
#define AURA_CHUNK 12
#endif
#ifndef AURA_PREP_WPE
#define AURA_PREP_WPE 4
#endif
constexpr int kChunkSteps = AURA_CHUNK;        // k-steps of the weight matrix held in LDS
constexpr int kChunk = kChunkSteps * kStepCells;
constexpr int kPitch = kChunk + 8;             // row pitch in 16-bit elements (rows start 4 banks apart)
constexpr int kHalf = 128;                     // channels of one half wave's row piece: 32 lanes x 4 channels
constexpr int kWinSide = 32;                   // side of the per-view cell map: one 32-bit word per row

static_assert(kSlots * kTilePts == kPrepThreads && kNIT * kSlots == kViewBatch, "thread mapping");
static_assert(sizeof(TileStep) == 64 + 2048, "k-step layout");

template <int DT>
__device__ __forceinline__ void split_weight(float w, uint16_t& hi, uint16_t& lo) {
  if constexpr (DT == 1) {
    __bf16 h = (__bf16)w;
    __bf16 l = (__bf16)(w - (float)h);
    hi = __builtin_bit_cast(uint16_t, h);
    lo = __builtin_bit_cast(uint16_t, l);
  } else {
    _Float16 h = (_Float16)w;
    _Float16 l = (_Float16)(w - (float)h);
    hi = __builtin_bit_cast(uint16_t, h);
    lo = __builtin_bit_cast(uint16_t, l);
  }
}

// ---- half-wave reductions on the data-parallel-primitive lanes: after the call, lane 31 holds
// the result over lanes 0..31 and lane 63 the result over lanes 32..63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ s16x2 dpp_pull(s16x2 identity, s16x2 v) {
  return __builtin_bit_cast(s16x2, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity), __builtin_bit_cast(int, v),
                                                                CTRL, ROW_MASK, 0xf, false));
}

template <bool IS_MIN>
__device__ __forceinline__ s16x2 half_wave_reduce(s16x2 v) {
  const s16x2 id = IS_MIN ? s16x2{0x7fff, 0x7fff} : s16x2{-0x8000, -0x8000};
#define AURA_RED_STEP(ctrl, mask)                                                                  \
  v = IS_MIN ? __builtin_elementwise_min(v, dpp_pull<ctrl, mask>(id, v)) : __builtin_elementwise_max(v, dpp_pull<ctrl, mask>(id, v))
  AURA_RED_STEP(0x111, 0xf);   // row_shr:1
  AURA_RED_STEP(0x112, 0xf);   // row_shr:2
  AURA_RED_STEP(0x114, 0xf);   // row_shr:4
  AURA_RED_STEP(0x118, 0xf);   // row_shr:8  -> lane 15 of every row of 16 holds the row's result
  AURA_RED_STEP(0x142, 0xa);   // row_bcast:15 into rows 1 and 3
#undef AURA_RED_STEP
  return v;
}

// Sum over each half of the wave with lane-shift adds (no LDS traffic): lanes 31 and 63 hold the sums.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}

template <int CTRL>
__device__ __forceinline__ int row_shift_add(int v) {
  return v + __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}

__device__ __forceinline__ float half_wave_sum(float v) {
  v = dpp_add<0x111, 0xf>(v);   // row_shr:1
  v = dpp_add<0x112, 0xf>(v);   // row_shr:2
  v = dpp_add<0x114, 0xf>(v);   // row_shr:4
  v = dpp_add<0x118, 0xf>(v);   // row_shr:8  -> lane 15 of every row of 16 holds the row's sum
  v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  return v;
}

// One (point, view) pair after Eq. 1 and the cell selection.
struct PairRec {
  int xy;        // y0 << 16 | x0 of the first cell, -1: the view does not see the point
  float ax, ay;  // weights of the second cell per axis
};

// The slow way out when a tile needs more k-steps than it owns: the workgroup fuses its 32 points by a
// per-point gather (wave per point, lanes over channels, 512 channels per sweep, the whole row in registers).
// The row is stored when the call has a place for it (FuseArgs::fused); when the call wants scores as well
// (FuseArgs::scoring), they are taken here from the row in registers, so that no later kernel needs the row:
// omega_k by a wave-wide sum per material, then Eq. 4 and the label with lanes over the materials.
constexpr int kGatherSweeps = 3;   // 512 channels each: D <= 1536 on this path

template <int DT>
__device__ __forceinline__ void gather_tile(const FuseArgs& a, const ObjRange& ob, int li0, int wave, int n_waves, int lane) {
  const int D = a.feat.D, Hf = a.feat.Hf, Wf = a.feat.Wf;
  const long long view_bytes = (long long)Hf * Wf * D * 2;
  for (int k = 0; k < kTilePts / n_waves; ++k) {
    const int li = li0 + wave * (kTilePts / n_waves) + k;
    if (li >= ob.n_pts) break;
    const long long i = ob.pt_begin + li;
    const float x = a.xyz[3 * i], y = a.xyz[3 * i + 1], z = a.xyz[3 * i + 2];
    float acc[kGatherSweeps][8];
#pragma unroll
    for (int s = 0; s < kGatherSweeps; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[s][e] = 0.0f;
    int cnt = 0;
    for (int vb = 0; vb < ob.n_views; vb += kWave) {
      bool seen = false;
      int x0 = 0, y0 = 0;
      float ax = 0.0f, ay = 0.0f;
      if (vb + lane < ob.n_views) {
        const int v = ob.view_begin + vb + lane;
        const Proj p = project(a.vis.cam + (long long)v * 16, x, y, z);
        const float* dv = a.vis.depth ? a.vis.depth + (long long)v * a.vis.H * a.vis.W : nullptr;
        seen = visible(a.vis, dv, p) && view_kept(a, i, vb + lane);
        if (a.out_vis) a.out_vis[i * a.vis_pitch + vb + lane] = seen ? 1 : 0;
        if (seen) {
          const Tap tx = tap_axis(p.u, a.feat.pitch_x, Wf), ty = tap_axis(p.v, a.feat.pitch_y, Hf);
          x0 = tx.i0; ax = tx.a;
          y0 = ty.i0; ay = ty.a;
        }
      }
      unsigned long long m = __ballot(seen);
      cnt += __popcll(m);
      while (m) {
        const int src = __builtin_ctzll(m);
        m &= m - 1;
        const int sx0 = __builtin_amdgcn_readlane(x0, src), sy0 = __builtin_amdgcn_readlane(y0, src);
        const float sax = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ax), src));
        const float say = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ay), src));
        const int sx1 = sx0 + 1 < Wf ? sx0 + 1 : Wf - 1, sy1 = sy0 + 1 < Hf ? sy0 + 1 : Hf - 1;
        const float wgt[4] = {(1.0f - sax) * (1.0f - say), sax * (1.0f - say), (1.0f - sax) * say, sax * say};
        const int cell[4] = {sy0 * Wf + sx0, sy0 * Wf + sx1, sy1 * Wf + sx0, sy1 * Wf + sx1};
        const char* vbase = static_cast<const char*>(a.feat.feat) + (long long)(ob.view_begin + vb + src) * view_bytes;
#pragma unroll
        for (int s = 0; s < kGatherSweeps; ++s) {
          const int ch = s * 8 * kWave + 8 * lane;
          if (ch < D) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const u32x4 raw = *reinterpret_cast<const u32x4*>(vbase + ((long long)cell[c] * D + ch) * 2);
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                float lo, hi;
                if constexpr (DT == 1) {
                  lo = __uint_as_float(raw[j] << 16);
                  hi = __uint_as_float(raw[j] & 0xffff0000u);
                } else {
                  lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(raw[j] & 0xffffu));
                  hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(raw[j] >> 16));
                }
                acc[s][2 * j] = __builtin_fmaf(wgt[c], lo, acc[s][2 * j]);
                acc[s][2 * j + 1] = __builtin_fmaf(wgt[c], hi, acc[s][2 * j + 1]);
              }
            }
          }
        }
      }
    }
    // mean over the visible views (Eq. 2), then the L2 normalisation
    const float inv = cnt > 0 ? 1.0f / (float)cnt : 0.0f;
    float ss = 0.0f;
#pragma unroll
    for (int s = 0; s < kGatherSweeps; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc[s][e] *= inv;
        ss = __builtin_fmaf(acc[s][e], acc[s][e], ss);
      }
    if (!a.mean_only) {
      const float scale = 1.0f / fmaxf(sqrtf(wave_sum(ss)), a.norm_eps);
#pragma unroll
      for (int s = 0; s < kGatherSweeps; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[s][e] *= scale;
    }
    if (a.fused) {
      float* __restrict__ out_row = a.fused + i * D;
#pragma unroll
      for (int s = 0; s < kGatherSweeps; ++s) {
        const int ch = s * 8 * kWave + 8 * lane;
        if (ch < D) {
          *reinterpret_cast<f32x4*>(out_row + ch) = f32x4{acc[s][0], acc[s][1], acc[s][2], acc[s][3]};
          *reinterpret_cast<f32x4*>(out_row + ch + 4) = f32x4{acc[s][4], acc[s][5], acc[s][6], acc[s][7]};
        }
      }
    }
    if (a.out_count && lane == 0) a.out_count[i] = cnt;

    if (a.scoring.G) {
      // Sec. 3.4.1 for this point: lane l keeps the similarities of materials l and l + 64
      const TileScoring& sc = a.scoring;
      float mine[2] = {-INFINITY, -INFINITY};
      for (int m = 0; m < sc.K; ++m) {
        const float* __restrict__ t = sc.temb + (long long)m * D;
        float dot = 0.0f;
#pragma unroll
        for (int s = 0; s < kGatherSweeps; ++s) {
          const int ch = s * 8 * kWave + 8 * lane;
          if (ch < D) {
            const f32x4 t0 = *reinterpret_cast<const f32x4*>(t + ch), t1 = *reinterpret_cast<const f32x4*>(t + ch + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              dot = __builtin_fmaf(acc[s][e], t0[e], dot);
              dot = __builtin_fmaf(acc[s][4 + e], t1[e], dot);
            }
          }
        }
        dot = wave_sum(dot);
        if ((m & 63) == lane) mine[m >> 6] = dot;
      }
      float best = fmaxf(mine[0], mine[1]);
      int bidx = mine[1] > mine[0] ? lane + 64 : lane;   // a lane without a material holds -inf
#pragma unroll
      for (int o = kWave / 2; o > 0; o >>= 1) {
        const float ob_ = __shfl_xor(best, o, kWave);
        const int oi = __shfl_xor(bidx, o, kWave);
        if (ob_ > best || (ob_ == best && oi < bidx)) { best = ob_; bidx = oi; }   // lowest index wins ties
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int m = lane + 64 * h;
        if (m < sc.K) sc.scores[i * sc.K + m] = mine[h];
      }
      if (sc.label && lane == 0) sc.label[i] = bidx;
      if (sc.prop) {
        float e[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) e[h] = lane + 64 * h < sc.K ? weight_exp((mine[h] - best) * sc.inv_T) : 0.0f;
        const float den = wave_sum(e[0] + e[1]);
        // all similarities exactly zero (nobody sees the point): zero properties where the caller asks for that
        const bool zero_row = sc.unseen_zero && __ballot((lane < sc.K && mine[0] != 0.0f) || (lane + 64 < sc.K && mine[1] != 0.0f)) == 0;
        for (int p = 0; p < sc.P; ++p) {
          float num = 0.0f;
#pragma unroll
          for (int h = 0; h < 2; ++h)
            if (lane + 64 * h < sc.K) num = __builtin_fmaf(e[h], sc.y[(lane + 64 * h) * sc.P + p], num);
          num = wave_sum(num);
          if (lane == 0) sc.prop[i * sc.P + p] = zero_row ? 0.0f : num / den;
        }
      }
    }
  }
}

// DT: 1 bf16, 2 fp16 feature maps (decides the 16-bit format of the weights).  SEL: the views of each point are
// given (FuseArgs::in_mask) instead of decided by the depth test; a variant of its own so that the usual path does
// not carry the test.
template <int DT, bool SEL>
__global__ __launch_bounds__(kPrepThreads) __attribute__((amdgpu_waves_per_eu(AURA_PREP_WPE)))
void k_tile_prepare(FuseArgs a, TileWs ws, ObjTable tab) {
  __shared__ int s_win[kViewBatch][2];                 // first cell (x, y) of the view's map
  __shared__ int s_mode[kViewBatch];                   // 0 nothing seen, 1 cell map, 2 private entries
  __shared__ uint32_t s_vmask[kViewBatch];             // which of the 32 points the view sees
  __shared__ __attribute__((aligned(16))) uint32_t s_bits[kViewBatch][kWinSide];   // map of touched cells, row = word
  __shared__ __attribute__((aligned(16))) uint16_t s_wbase[kViewBatch][kWinSide];  // set bits before each row
  __shared__ int s_base[kViewBatch + 1];               // first list index of each view
  __shared__ __attribute__((aligned(16))) uint32_t s_cell[kChunk];
  __shared__ __attribute__((aligned(16))) uint16_t s_whi[kTilePts][kPitch];
  __shared__ __attribute__((aligned(16))) uint16_t s_wlo[kTilePts][kPitch];
  __shared__ int s_cnt[kTilePts];

  const ObjRange ob = tab.o[blockIdx.y];
  const int nblk = (ob.n_pts + kTilePts - 1) / kTilePts;
  if ((int)blockIdx.x >= nblk) return;
  const int blk = xcd_contiguous(blockIdx.x, nblk);
  TileHdr* __restrict__ hdr = ws.hdr + ob.tile_begin + blk;
  const long long slot0 = (long long)(ob.tile_begin + blk) * ws.quota;   // first k-step the tile owns
  const int tid = threadIdx.x, lane = tid % kWave;
  const int Hf = a.feat.Hf, Wf = a.feat.Wf;
  const uint32_t row_bytes = (uint32_t)a.feat.D * 2u;
  const int p = tid % kTilePts;          // point of this thread
  const int slot = tid / kTilePts;       // view slot of this thread
  const int li0 = blk * kTilePts;
  const bool p_valid = li0 + p < ob.n_pts;
  const long long ip = ob.pt_begin + li0 + (p_valid ? p : 0);
  const float px = a.xyz[3 * ip], py = a.xyz[3 * ip + 1], pz = a.xyz[3 * ip + 2];

  if (tid < kTilePts) s_cnt[tid] = 0;
  if (blockIdx.x == 0 && tid < 8) ws.counters[(ws.obj_base + blockIdx.y) * 8 + tid] = 0u;   // for the product kernel
  int used = 0;   // k-steps written so far (the view batches follow one another in the tile's run)
  bool exhausted = false;

  for (int vb0 = 0; vb0 < ob.n_views; vb0 += kViewBatch) {
    const int nvb = min(kViewBatch, ob.n_views - vb0);
    __syncthreads();   // the previous batch is done with the tables (and s_cnt is initialised)
    *reinterpret_cast<u32x4*>(&s_bits[tid / 8][4 * (tid % 8)]) = u32x4{0u, 0u, 0u, 0u};

    // ---- A: project and test; bounding box of the touched cells per view
    PairRec pr[kNIT];
    int my_cnt = 0;
    // All projections of the batch first, then all depth texels, then the tests: a thread's four pairs are four chains
    // of camera row -> projection -> texel address -> texel, and in one loop each chain waited for the one before it
    // (11 K of a tile's 26 K cycles with 32 views).
    Proj pjs[kNIT];
    bool frs[kNIT];
    float deps[kNIT];
#pragma unroll
    for (int it = 0; it < kNIT; ++it) {
      const int v = ob.view_begin + vb0 + min(it * kSlots + slot, nvb - 1);   // (a slot beyond the batch: its last view again)
      pjs[it] = project(a.vis.cam + (long long)v * 16, px, py, pz);
      frs[it] = in_frustum(a.vis, pjs[it]);
    }
#pragma unroll
    for (int it = 0; it < kNIT; ++it) {
      const int v = ob.view_begin + vb0 + min(it * kSlots + slot, nvb - 1);
      deps[it] = 1.0f;
      if (a.vis.depth) deps[it] = a.vis.depth[(long long)v * a.vis.H * a.vis.W + (frs[it] ? depth_texel(a.vis, pjs[it]) : 0)];
    }
#pragma unroll
    for (int it = 0; it < kNIT; ++it) {
      pr[it].xy = -1;
      pr[it].ax = pr[it].ay = 0.0f;
      if (it * kSlots >= nvb) continue;   // uniform
      const int vl = it * kSlots + slot;
      const Proj pj = pjs[it];
      const bool fr = frs[it];
      const float dep = deps[it];
      bool seen = vl < nvb && p_valid && fr && (a.vis.frustum_only || passes_depth(a.vis, pj, dep));
      if constexpr (SEL) seen = seen && view_kept(a, ip, vb0 + min(vl, nvb - 1));
      s16x2 lo2 = {0x7fff, 0x7fff}, hi2 = {-1, -1};   // (x, y) of the first / second cell
      if (seen) {
        const Tap tx = tap_axis(pj.u, a.feat.pitch_x, Wf), ty = tap_axis(pj.v, a.feat.pitch_y, Hf);
        pr[it].ax = tx.a;
        pr[it].ay = ty.a;
        pr[it].xy = (ty.i0 << 16) | tx.i0;
        lo2 = s16x2{(short)tx.i0, (short)ty.i0};
        hi2 = s16x2{(short)tx.i1, (short)ty.i1};
        ++my_cnt;
      }
      const unsigned long long seen_mask = __ballot(seen);
      lo2 = half_wave_reduce<true>(lo2);
      hi2 = half_wave_reduce<false>(hi2);
      if (p == kTilePts - 1 && vl < nvb) {
        const bool any = hi2[0] >= 0;
        const int ww = hi2[0] - lo2[0] + 1, wh = hi2[1] - lo2[1] + 1;
        s_win[vl][0] = lo2[0];
        s_win[vl][1] = lo2[1];
        s_mode[vl] = !any ? 0 : (ww <= kWinSide && wh <= kWinSide ? 1 : 2);
        s_vmask[vl] = (uint32_t)(seen_mask >> (lane & 32));
      }
    }
    if (my_cnt) atomicAdd(&s_cnt[p], my_cnt);
    __syncthreads();
    if (a.out_vis && tid < kTilePts && p_valid) {
      // the mask of Eq. 1 for this batch of views, from the per-view bit masks: point tid's bytes, four per store
      // where the row pitch allows
      uint8_t* __restrict__ vrow = a.out_vis + (ob.pt_begin + li0 + tid) * a.vis_pitch + vb0;
      if ((a.vis_pitch & 3) == 0) {
        for (int v4 = 0; v4 < nvb; v4 += 4) {
          uint32_t w = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (v4 + e < nvb) w |= ((s_vmask[v4 + e] >> tid) & 1u) << (8 * e);
          if (v4 + 4 <= nvb) {
            *reinterpret_cast<uint32_t*>(vrow + v4) = w;
          } else {
            for (int e = 0; v4 + e < nvb; ++e) vrow[v4 + e] = (uint8_t)((w >> (8 * e)) & 1u);
          }
        }
      } else {
        for (int v = 0; v < nvb; ++v) vrow[v] = (uint8_t)((s_vmask[v] >> tid) & 1u);
      }
    }

    // ---- B: mark the touched cells of every view that uses a map
#pragma unroll
    for (int it = 0; it < kNIT; ++it) {
      if (pr[it].xy < 0) continue;
      const int vl = it * kSlots + slot;
      if (s_mode[vl] != 1) continue;
      const int x0 = pr[it].xy & 0xffff, y0 = pr[it].xy >> 16;
      const int bit = (y0 - s_win[vl][1]) * kWinSide + (x0 - s_win[vl][0]);
      const bool has_x1 = x0 + 1 < Wf, has_y1 = y0 + 1 < Hf;   // at the border the second cell has weight 0
      atomicOr(&s_bits[vl][bit >> 5], 1u << (bit & 31));
      if (has_x1) atomicOr(&s_bits[vl][(bit + 1) >> 5], 1u << ((bit + 1) & 31));
      if (has_y1) atomicOr(&s_bits[vl][(bit + kWinSide) >> 5], 1u << ((bit + kWinSide) & 31));
      if (has_x1 && has_y1) atomicOr(&s_bits[vl][(bit + kWinSide + 1) >> 5], 1u << ((bit + kWinSide + 1) & 31));
    }
    __syncthreads();
    if (tid < kWave) {   // list length of every view, exclusive scan over the views
      int n = 0;
      if (lane < nvb) {
        if (s_mode[lane] == 1) {
#pragma unroll 8
          for (int w = 0; w < kWinSide; ++w) {
            s_wbase[lane][w] = (uint16_t)n;
            n += __popc(s_bits[lane][w]);
          }
        } else if (s_mode[lane] == 2) {
          n = 4 * __popc(s_vmask[lane]);
        }
      }
      int inc = n;
#pragma unroll
      for (int o = 1; o < kViewBatch; o <<= 1) {
        const int up = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += up;
      }
      if (lane < kViewBatch) s_base[lane] = inc - n;
      if (lane == kViewBatch - 1) s_base[kViewBatch] = inc;
    }
    __syncthreads();
    const int L = s_base[kViewBatch];
    const int nsteps = (L + kStepCells - 1) / kStepCells;
    if (used + nsteps > ws.quota) {   // uniform
      exhausted = true;
      break;
    }
    const int off = used;
    used += nsteps;

    // ---- C: chunks of the list -> weight matrix in LDS -> k-steps in global memory
    for (int c0 = 0; c0 < L; c0 += kChunk) {
      const int Lc = min(kChunk, L - c0);
      const int ksteps = (Lc + kStepCells - 1) / kStepCells;
      if (c0 > 0) __syncthreads();   // the previous chunk has been copied out
      for (int q = tid; q < kTilePts * ksteps * 2; q += kPrepThreads) {   // zero the matrix, 16 bytes per store
        const int row = q / (ksteps * 2), col = (q % (ksteps * 2)) * 8;
        const u32x4 z = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(&s_whi[row][col]) = z;
        *reinterpret_cast<u32x4*>(&s_wlo[row][col]) = z;
      }
      // entries that pad the last k-step point at a cell that exists (their weights are zero)
      if (tid >= Lc && tid < ksteps * kStepCells) s_cell[tid] = (uint32_t)((ob.view_begin + vb0) * Hf * Wf) * row_bytes;
      __syncthreads();
      // weights and cells of every visible pair (a cell that several points touch gets the same value from each of
      // them; walking over the set bits of the maps instead kept a few threads busy for 4 K of a tile's 25 K cycles)
#pragma unroll
      for (int it = 0; it < kNIT; ++it) {
        if (pr[it].xy < 0) continue;
        const int vl = it * kSlots + slot;
        const int x0 = pr[it].xy & 0xffff, y0 = pr[it].xy >> 16;
        const float ax = pr[it].ax, ay = pr[it].ay;
        const bool has_x1 = x0 + 1 < Wf, has_y1 = y0 + 1 < Hf;
        const float wgt[4] = {(1.0f - ax) * (1.0f - ay), ax * (1.0f - ay), (1.0f - ax) * ay, ax * ay};
        const bool on[4] = {true, has_x1, has_y1, has_x1 && has_y1};
        int idx[4];
        if (s_mode[vl] == 1) {
          const int bit = (y0 - s_win[vl][1]) * kWinSide + (x0 - s_win[vl][0]);
          const int bs[4] = {bit, bit + 1, bit + kWinSide, bit + kWinSide + 1};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int b = on[k] ? bs[k] : bit;
            idx[k] = s_base[vl] + s_wbase[vl][b >> 5] + __popc(s_bits[vl][b >> 5] & ((1u << (b & 31)) - 1u)) - c0;
            if (on[k] && idx[k] >= 0 && idx[k] < Lc)
              s_cell[idx[k]] = (uint32_t)(((ob.view_begin + vb0 + vl) * Hf + y0 + (k >> 1)) * Wf + x0 + (k & 1)) * row_bytes;
          }
        } else {
          const int first = s_base[vl] + 4 * __popc(s_vmask[vl] & ((1u << p) - 1u)) - c0;
          const int cell0 = (ob.view_begin + vb0 + vl) * Hf;
          const int x1 = has_x1 ? x0 + 1 : x0, y1 = has_y1 ? y0 + 1 : y0;
          const int cx[4] = {x0, x1, x0, x1}, cy[4] = {y0, y0, y1, y1};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            idx[k] = first + k;
            if (idx[k] >= 0 && idx[k] < Lc) s_cell[idx[k]] = (uint32_t)((cell0 + cy[k]) * Wf + cx[k]) * row_bytes;
          }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if (on[k] && idx[k] >= 0 && idx[k] < Lc) {
            uint16_t hi, lo;
            split_weight<DT>(wgt[k], hi, lo);
            s_whi[p][idx[k]] = hi;
            s_wlo[p][idx[k]] = lo;
          }
        }
      }
      __syncthreads();
      // copy out: per k-step 16 cell offsets and the two operand matrices (64 lanes x 16 bytes each)
      TileStep* __restrict__ out = ws.steps + slot0 + off + c0 / kStepCells;
      for (int q = tid; q < ksteps * 128; q += kPrepThreads) {
        const int s = q >> 7, part = (q >> 6) & 1, l = q & 63, g = l >> 5, m = l & 31;
        const uint16_t* src = part ? &s_wlo[m][kStepCells * s + 8 * g] : &s_whi[m][kStepCells * s + 8 * g];
        const u32x4 val = *reinterpret_cast<const u32x4*>(src);
        u32x4* dst = part ? &out[s].a_lo[l] : &out[s].a_hi[l];
        *reinterpret_cast<u32x4*>(dst) = val;
      }
      if (tid < ksteps * kStepCells) out[tid / kStepCells].cell[tid % kStepCells] = s_cell[tid];
    }
  }

  if (a.out_vis && tid < kTilePts && li0 + tid < ob.n_pts) {   // mask columns beyond the object's views
    for (int j = ob.n_views; j < a.vis_pitch; ++j) a.out_vis[(ob.pt_begin + li0 + tid) * a.vis_pitch + j] = 0;
  }
  __syncthreads();
  if (exhausted) {
    if (tid == 0) {
      hdr->nsteps = -1;
      atomicAdd(ws.status + 1, 1u);   // second status word: tiles fused by the gather
    }
    gather_tile<DT>(a, ob, li0, tid / kWave, kPrepThreads / kWave, lane);
    return;
  }
  if (tid == 0) hdr->nsteps = used;
  if (tid < kTilePts) {
    hdr->cnt[tid] = s_cnt[tid];
    if (a.out_count && li0 + tid < ob.n_pts) a.out_count[ob.pt_begin + li0 + tid] = s_cnt[tid];
  }
}

// ------------------------------------------------------------------------------------ product

template <int DT>
__device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c) {
  if constexpr (DT == 1)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Operands of one k-step in registers: the two weight operands, the lane's 8 cell offsets, and
// 8 cell rows.
struct StepA {
  u32x4 hi, lo;
};

struct StepC {
  u32x4 lo, hi;   // byte offsets of the lane's cells: 8 g .. 8 g + 3 and 8 g + 4 .. 8 g + 7
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int H>
struct StepQ {
  u32x2 q[H][8];   // [128-channel piece of the wave's span][cell]: 4 channels each
};

// What the prepare kernel wrote is constant for the product kernel: reading the tile header
// through the constant address space keeps the wave-uniform read on the scalar unit even inside
// the tile loop, where the compiler must otherwise assume that the stores of fused rows alias it.
typedef const uint32_t __attribute__((address_space(4))) * const_words;

__device__ __forceinline__ int load_nsteps(const TileHdr* h) {
  return (int)((const_words)(uintptr_t)&h->nsteps)[0];
}

// A tile's k-steps are staged in LDS before they are used (two buffers of kStage k-steps): the
// weight operands were written by the prepare kernel and come from far memory, the copy for the
// next tile is issued when the current tile starts and is hidden behind it.  The copy is a
// direct global -> LDS load (no registers): one instruction moves 64 x 16 contiguous bytes.
//
// The copy instruction is written as inline assembly on purpose.  Issued through the compiler's
// builtin, a copy that is still in flight makes every later wait for a vector read a wait for ALL
// outstanding reads (the compiler cannot tell which LDS reads the copy may feed), which serialises
// the row reads of the product loop.  Hidden from that bookkeeping, the copies only make the
// hardware counter larger than the compiler assumes; reads complete in order, so its waits remain
// sufficient.  The workgroup waits for the copies explicitly (wait_copies) before the barrier that
// publishes a buffer.
template <int S>
constexpr int stage_steps_for() { return S == 1 ? 4 : (S == 2 ? 8 : 16); }   // S: units of 256 channels   // keeps 8 waves per compute unit in LDS

__device__ __forceinline__ void copy_64x16(const char* g, char* lds) {
  // m0 = LDS byte address of the 1 KiB piece; lane l's 16 bytes land at m0 + 16 l
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds);
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0) : "s"(lds_addr), "v"(g) : "memory");
}

__device__ __forceinline__ void wait_copies() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int S>
__device__ __forceinline__ void stage_steps(char* lds, const TileStep* __restrict__ src, int nsteps, int span, int lane) {
  const int bytes = nsteps * (int)sizeof(TileStep);
  const char* g = reinterpret_cast<const char*>(src);
  for (int piece = span; piece * 1024 < bytes; piece += S) {
    const int off = piece * 1024 + lane * 16;
    if (off < bytes) copy_64x16(g + off, lds + piece * 1024);
  }
}

__device__ __forceinline__ void lds_a(const char* lds, int k, int lane, StepA& r) {
  const TileStep* st = reinterpret_cast<const TileStep*>(lds) + k;
  r.hi = st->a_hi[lane];
  r.lo = st->a_lo[lane];
}

__device__ __forceinline__ void lds_c(const char* lds, int k, int g, StepC& r) {
  const TileStep* st = reinterpret_cast<const TileStep*>(lds) + k;
  r.lo = *reinterpret_cast<const u32x4*>(&st->cell[8 * g]);
  r.hi = *reinterpret_cast<const u32x4*>(&st->cell[8 * g + 4]);
}

template <int H>
__device__ __forceinline__ void load_q(const char* __restrict__ feat, const StepC& c, uint32_t lane_off, StepQ<H>& r) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t cell = e < 4 ? c.lo[e] : c.hi[e - 4];
#pragma unroll
    for (int h = 0; h < H; ++h) r.q[h][e] = *reinterpret_cast<const u32x2*>(feat + (cell + lane_off + h * kHalf * 2));
  }
}

// The matrix-core instructions of one k-step: operand t = 4 h + j holds channel 128 h + 4 m + j of
// the 8 cells.
template <int DT, int H>
__device__ __forceinline__ void mma_step(const StepA& w, const StepQ<H>& r, f32x16 (&acc)[4 * H]) {
#pragma unroll
  for (int t = 0; t < 4 * H; ++t) {
    u32x4 b;
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      // bytes 0..3 of the selector index the first cell's dword, 4..7 the second cell's
      const uint32_t lo = r.q[t >> 2][2 * e2][(t >> 1) & 1], hi = r.q[t >> 2][2 * e2 + 1][(t >> 1) & 1];
      b[e2] = __builtin_amdgcn_perm(hi, lo, (t & 1) ? 0x07060302u : 0x05040100u);
    }
    acc[t] = mma<DT>(w.hi, b, acc[t]);
    acc[t] = mma<DT>(w.lo, b, acc[t]);
  }
}

struct ProdArgs {
  const char* feat;
  int D;
  const TileHdr* hdr;
  const TileStep* steps;
  unsigned* counters;   // [objects of the launch][8]
  int quota;
  float* fused;
  float* factor;        // [N] or nullptr: what each point's raw tile product was multiplied by
  float norm_eps;
  int mean_only;
};

// DT: 1 bf16, 2 fp16 feature maps.  S waves per workgroup, each owning H pieces of 128 channels:
// D == 128 * H * S.  PF: k-steps whose cell rows are requested ahead of their products.
//
// A workgroup walks over several tiles.  While a tile is multiplied, the k-steps of the next one
// are copied into the other LDS buffer; per k-step the weight operands and cell offsets come from
// LDS and the cell rows (shared with the neighbouring tiles, so mostly L2 hits) are read PF
// k-steps ahead of their product.  The k-steps are taken in groups of PF without a branch inside, so
// that the wait counters before each product allow for exactly the reads issued after its operands.
// A tile has one barrier (after its products); nothing in the tile loop waits for a round trip to memory
// that was started in the same tile:
//   * the ticket of a tile (see below) is asked for three tiles ahead,
//   * the length of its list is read two tiles ahead (a vector read: a scalar read would share its
//     counter with the LDS reads and stall them),
//   * its k-steps are copied one tile ahead,
//   * its first rows are requested right after the previous tile's stores.
// Memory operations inside the loop are unconditional (reads for a tile that does not exist go to cell 0,
// stores of rows that do not exist are dropped by the buffer bounds check): behind a branch the compiler
// has to assume the worst about outstanding operations and waits for all of them.
//
// Tile order: the workgroups with the same id modulo 8 run on the same XCD; XCD c owns one
// contiguous range of the object's tiles and its workgroups take the next tile of that range from
// a counter (tiles differ in length, a fixed split leaves a tail), so that at any time the tiles in
// flight on an XCD are neighbours and share cell rows in its L2.
constexpr int kXcd = 8;
constexpr int kFusedGroupsMax = 512;  // one-kernel form: two workgroups per compute unit
constexpr int kProdGroupsMax = 768;   // two workgroups fit a compute unit at a time; the rest take over as the first run out of tiles

// The opening reads of a tile whose k-steps are staged at `sb` (n of them, possibly none): the rows of its
// first PF k-steps and the weights of its first k-step.  With nothing staged the reads go to cell 0 and are
// not used.
template <int H, int PF>
__device__ __forceinline__ void open_tile(const char* sb, int n_staged, const char* __restrict__ feat, uint32_t lane_off,
                                          int lane, int g, StepA (&wa)[2], StepQ<H> (&rq)[PF]) {
  const uint32_t on = n_staged > 0 ? 0xffffffffu : 0u;
  const int l0 = max(n_staged - 1, 0);
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    StepC c;
    lds_c(sb, min(j, l0), g, c);
    c.lo &= on;
    c.hi &= on;
    load_q(feat, c, lane_off, rq[j]);
  }
  lds_a(sb, 0, lane, wa[0]);
}

// Which of an object's tiles an XCD works on, in the order of its tickets.  The tiles go to the XCDs in chunks of
// consecutive tiles taken in turn (ticket t of XCD x is tile ((t / chunk) * 8 + x) * chunk + t % chunk): neighbouring
// tiles still meet in one L2, and every XCD gets a sample of the whole object instead of one contiguous eighth, whose
// k-steps per tile can differ (1 M points on six ellipsoids, 32 views: the eighths finished between 665 and 775 us).
// The tiles behind the last whole round of chunks are split into eight contiguous parts, so that the XCDs' shares
// differ by one tile at most and the first XCDs hold the larger ones (handed out as whole chunks, 6250 tiles gave two XCDs 832 and 810 tiles and the others 768).
struct XcdTiles {
  int sh, xcd_sh, full, rest_at, len;   // chunk = 2^sh; tickets below `full` are chunked, the others contiguous
  __device__ XcdTiles(int nblk, int xcd) {
    sh = 31 - __builtin_clz(max(1, min(64, nblk / (8 * kXcd))));   // chunk = 2^sh tiles: 64, fewer for small objects
    const int rounds = nblk >> (sh + 3);                            // kXcd = 8 chunks per round
    static_assert(kXcd == 8, "rounds of eight chunks");
    full = rounds << sh;
    const int base = rounds << (sh + 3), rest = nblk - base;
    // XCD x takes rest / 8 of them and one more while x < rest % 8: an object of fewer than eight tiles has workgroups on
    // its first XCDs only
    const int q = rest >> 3, extra = rest & 7;
    rest_at = base + xcd * q + min(xcd, extra) - full;
    len = full + q + (xcd < extra ? 1 : 0);
    xcd_sh = xcd << sh;
  }
  __device__ int at(int t) const {
    return t < full ? ((((t >> sh) * kXcd) << sh) + xcd_sh + (t & ((1 << sh) - 1))) : rest_at + t;
  }
};

template <int DT, int S, int H, int PF>
__global__ __launch_bounds__(kWave* S) __attribute__((amdgpu_waves_per_eu(H == 1 ? 3 : 2, H == 1 ? 3 : 2)))
void k_tile_product(ProdArgs a, ObjTable tab) {
  constexpr int kSpan = kHalf * H;   // channels per wave
  constexpr int kStage = stage_steps_for<S * H / 2>();
  __shared__ __attribute__((aligned(16))) char s_steps[2][kStage * sizeof(TileStep)];
  __shared__ float s_ss[2][S][kTilePts];   // [tile parity]: a wave may write the next tile's sums while another still reads
  __shared__ int s_take[2];

  const ObjRange ob = tab.o[blockIdx.y];
  const int nblk = (ob.n_pts + kTilePts - 1) / kTilePts;
  const int groups = min(nblk, (int)gridDim.x);   // workgroups that work on this object
  if ((int)blockIdx.x >= groups) return;
  // The XCD's tiles and its counter (see XcdTiles: chunks of consecutive tiles taken in turn by the XCDs).
  const int xcd = blockIdx.x % kXcd;
  const XcdTiles mine(nblk, xcd);
  const int len = mine.len;
  auto tile_at = [&](int t) { return mine.at(t); };
  unsigned* __restrict__ ctr = a.counters + blockIdx.y * kXcd + xcd;
  const TileHdr* __restrict__ hdrs = a.hdr + ob.tile_begin;

  const int tid = threadIdx.x, lane = tid % kWave;
  const int span = __builtin_amdgcn_readfirstlane(tid / kWave);   // wave index: uniform, kept in a scalar register
  const int m = lane & 31, g = lane >> 5;
  const int D = a.D;
  const uint32_t lane_off = (uint32_t)(span * kSpan + 4 * m) * 2u;   // byte offset of the lane's first piece

  StepA wa[2];      // weight operands of the current and the next k-step
  StepC wc;         // cell offsets of the k-step whose rows are requested next
  StepQ<H> rq[PF];  // cell rows of the next PF k-steps

  // The first three tiles.  In the loop, a tile's ticket is asked for three tiles ahead, the length of its
  // list is read two tiles ahead and its k-steps are copied one tile ahead, so that none of the three
  // round trips is waited for.
  if (tid == 0) s_take[0] = (int)atomicAdd(ctr, 3u);
  __syncthreads();
  const int t0 = s_take[0];
  if (t0 >= len) return;
  int blk = tile_at(t0);
  int nxt = t0 + 1 < len ? tile_at(t0 + 1) : -1;    // -1: no further tile
  int nxt2 = t0 + 2 < len ? tile_at(t0 + 2) : -1;
  int buf = 0;
  int n = load_nsteps(hdrs + blk);
  int n_next = nxt >= 0 ? load_nsteps(hdrs + nxt) : 0;
  int pend_n = hdrs[max(nxt2, 0)].nsteps;   // list length of the tile after the next, picked up one tile later
  stage_steps<S>(s_steps[0], a.steps + (long long)(ob.tile_begin + blk) * a.quota, min(max(n, 0), kStage), span, lane);
  wait_copies();
  __syncthreads();
  open_tile<H, PF>(s_steps[0], min(max(n, 0), kStage), a.feat, lane_off, lane, g, wa, rq);

  while (blk >= 0) {
    const TileStep* __restrict__ st = a.steps + (long long)(ob.tile_begin + blk) * a.quota;
    // ask for the tile three tiles ahead (the answer is picked up after this tile's products)
    int asked = 0;
    if (tid == 0 && nxt2 >= 0) asked = (int)atomicAdd(ctr, 1u);
    // the next tile's k-steps go to the other buffer while this tile is multiplied
    stage_steps<S>(s_steps[buf ^ 1], a.steps + (long long)(ob.tile_begin + max(nxt, 0)) * a.quota,
                   nxt >= 0 ? min(max(n_next, 0), kStage) : 0, span, lane);
    const int my_cnt = hdrs[blk].cnt[tid % kTilePts];   // views that see point (lane % 32) of this tile

    f32x16 acc[4 * H];
#pragma unroll
    for (int t = 0; t < 4 * H; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

    const char* sb = s_steps[buf];
    for (int base = 0; base < n; base += kStage) {
      const int cnt = min(kStage, n - base), l0 = cnt - 1;
      if (base > 0) {
        // a tile with more k-steps than a buffer holds (rare): refill the buffer in place
        __syncthreads();
        stage_steps<S>(s_steps[buf], st + base, cnt, span, lane);
        wait_copies();
        __syncthreads();
        open_tile<H, PF>(sb, cnt, a.feat, lane_off, lane, g, wa, rq);
      }
      // k-steps in groups of PF without a branch inside: rows of k-step s + j + PF are requested right after
      // the products of k-step s + j have freed their registers (requests past the end repeat the last k-step)
      int s = 0;
      for (; s + PF <= cnt; s += PF) {
#pragma unroll
        for (int j = 0; j < PF; ++j) {
          lds_c(sb, min(s + j + PF, l0), g, wc);
          lds_a(sb, min(s + j + 1, l0), lane, wa[(j + 1) & 1]);
          mma_step<DT, H>(wa[j & 1], rq[j], acc);
          __builtin_amdgcn_sched_barrier(0);   // keep the reads behind the products that free their registers
          load_q(a.feat, wc, lane_off, rq[j]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // the last cnt - s < PF k-steps: their rows are there (or on the way), nothing more to request
#pragma unroll
      for (int j = 0; j < PF - 1; ++j) {
        if (s + j < cnt) {
          lds_a(sb, min(s + j + 1, l0), lane, wa[(j + 1) & 1]);
          mma_step<DT, H>(wa[j & 1], rq[j], acc);
        }
      }
    }

    // ---- sums of squares of the wave's channels, per point
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 8 * (r >> 2) + 4 * g + (r & 3);
      float ss = 0.0f;
#pragma unroll
      for (int t = 0; t < 4 * H; ++t) ss = __builtin_fmaf(acc[t][r], acc[t][r], ss);
      ss = half_wave_sum(ss);
      if (m == 31) s_ss[buf][span][row] = ss;
    }
    if (tid == 0) s_take[buf] = asked;
    const int n_next2 = __builtin_amdgcn_readfirstlane(pend_n);
    wait_copies();
    __syncthreads();   // the one barrier of a tile: sums, ticket and the next tile's k-steps are in LDS; every
                       // wave is done with this tile's buffer

    // the tile three ahead: its list length is requested now and read after the next tile's products
    const int t3 = s_take[buf];
    const int nxt3 = (nxt2 >= 0 && t3 < len) ? tile_at(t3) : -1;
    pend_n = hdrs[max(nxt3, 0)].nsteps;

    // ---- mean and L2 norm: one factor per point, inv_count / max(norm of the mean, eps), applied to the raw
    // sums.  Lane l of every wave computes the factor of point l % 32; a lane fetches the factors of its 16
    // rows from those lanes.
    float factor;
    {
      const float inv = my_cnt > 0 ? 1.0f / (float)my_cnt : 0.0f;
      float tot = 0.0f;
#pragma unroll
      for (int w = 0; w < S; ++w) tot += s_ss[buf][w][m];
      const float normed = inv / fmaxf(sqrtf(tot) * inv, a.norm_eps);
      factor = a.mean_only ? inv : normed;
    }
    {   // the factor of every point of the tile, for the scoring kernel (lanes 0..31 of the first wave; all
        // other lanes, and every lane when no factor array was given, fall outside the buffer)
      const int rows_f = a.factor ? min(kTilePts, ob.n_pts - blk * kTilePts) : 0;
      const __amdgpu_buffer_rsrc_t fout = __builtin_amdgcn_make_buffer_rsrc(a.factor + (a.factor ? ob.pt_begin + blk * kTilePts : 0), 0,
                                                                            rows_f * 4, 0x00020000);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_int(factor), fout, tid < kTilePts ? 4 * tid : 0x7ffffff0, 0, 0);
    }
    {
      // Buffer stores: the wave's part of the tile (rows of D floats, starting at a wave-uniform
      // address) is described by a buffer resource whose size covers the rows that exist, so a lane
      // only needs one 32-bit offset register and rows beyond the object's last point (or all rows, for
      // a tile that the prepare kernel fused itself: n < 0) are dropped by the bounds check instead of by
      // branches.
      const int li0 = blk * kTilePts;
      float* obase = a.fused ? a.fused + (ob.pt_begin + li0) * D + span * kSpan : nullptr;
      uint32_t row_bytes = (uint32_t)D * 4u;
      // opaque to the optimiser: otherwise the 32 per-row offsets below, which do not change from tile
      // to tile, are kept in registers across the whole tile loop and push other values into scratch
      asm volatile("" : "+s"(row_bytes));
      const int rows = (n >= 0 && a.fused) ? min(kTilePts, ob.n_pts - li0) : 0;   // no rows wanted: every store is dropped
      const __amdgpu_buffer_rsrc_t out = __builtin_amdgcn_make_buffer_rsrc(obase, 0, (int)(rows * row_bytes), 0x00020000);
      const uint32_t lane_out = (uint32_t)(4 * g) * row_bytes + (uint32_t)(4 * m) * 4u;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row0 = 8 * (r >> 2) + (r & 3);
        const float scale = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (row0 + 4 * g), __float_as_int(factor)));
#pragma unroll
        for (int h = 0; h < H; ++h) {
          const f32x4 v = {acc[4 * h][r] * scale, acc[4 * h + 1][r] * scale, acc[4 * h + 2][r] * scale, acc[4 * h + 3][r] * scale};
          // the scalar-offset operand stays 0: with a register there, a store directly followed by
          // an instruction that overwrites its data registers was seen to write stale lanes
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), out,
                                                 (int)(lane_out + (uint32_t)row0 * row_bytes) + h * kHalf * 4, 0, /*streaming*/ 2);
        }
      }
    }
    // The next tile's opening reads.  They are issued after the stores: the counter of outstanding memory
    // operations is in order, and with the stores behind them the compiler's wait before the first product
    // would cover every read at once instead of one k-step at a time.
    __builtin_amdgcn_sched_barrier(0);
    open_tile<H, PF>(s_steps[buf ^ 1], nxt >= 0 ? min(max(n_next, 0), kStage) : 0, a.feat, lane_off, lane, g, wa, rq);

    blk = nxt;
    nxt = nxt2;
    nxt2 = nxt3;
    n = n_next;
    n_next = n_next2;
    buf ^= 1;
  }
}

// ------------------------------------------------------------------------------------ one kernel
//
// k_tile_fused: the product kernel with one more wave per workgroup, the producer, that does the prepare kernel's work
// for the workgroup's NEXT tile while the S product waves multiply the current one.  The producer writes the k-steps
// straight into the other LDS buffer, in the layout the product waves read (no trip through memory, unless the scoring
// kernel wants them), so the projection -> depth read -> list -> weight chain of a tile hides behind the stores of the
// tile before it.  The tile's one barrier is shared: after it the buffer the products came from belongs to the producer
// and the buffer it filled belongs to the product waves.  The producer has no barrier of its own: it is one wave, and
// orders its LDS traffic with wave-level fences.  Tiles go to workgroups through the per-XCD counters as before; the
// producer asks for a ticket one tile ahead.  A tile whose list does not fit the buffer is fused by the producer itself
// (per-point gather): the launch code only takes this kernel where that is rare.

constexpr int kPBatch = 16;   // views per pass of the producer waves: two per trip, one per half wave
constexpr int kMaxProducers = 4;
constexpr int kCamRows = 32;  // camera rows of the object kept in LDS for the producer
constexpr int kOneKernelViews = 8;

typedef const float __attribute__((address_space(3))) * lds_floats;

struct ProducerScratch {
  uint32_t bits[kPBatch][kWinSide];   // map of touched cells per view, row = word
  uint16_t wbase[kPBatch][kWinSide];  // set bits before each row
  int base[kPBatch + 1];              // first list index of each view
  int win[kPBatch][2];
  int mode[kPBatch];
  uint32_t vmask[kPBatch];
};

struct TileSlot {    // what the product waves need to know about a staged tile
  int tile;          // index within the object; -1: no further tile
  int nsteps;        // -1: fused by the producers
  int pad_[2];
  int cnt[kMaxProducers][kTilePts];   // views that see each point, per producer wave
  uint32_t vmask[kCamRows];           // per view of the object: which of the tile's 32 points it sees (Eq. 1)
};

// Orders the producer wave's LDS traffic for the compiler.  The LDS unit handles the instructions of one wave in
// program order, so a later read by any lane sees an earlier write by any other lane of the same wave: no wait and
// no barrier instruction is needed, only that the compiler keeps the order.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// The point that lane `lane` of a producer wave handles in tile `blk` (lane % 32; the tile's first point where the
// object has no such point).
__device__ __forceinline__ float3 tile_point(const FuseArgs& a, const ObjRange& ob, int blk, int lane) {
  const int p = lane & 31, li0 = blk * kTilePts;
  const long long ip = ob.pt_begin + li0 + (li0 + p < ob.n_pts ? p : 0);
  return float3{a.xyz[3 * ip], a.xyz[3 * ip + 1], a.xyz[3 * ip + 2]};
}

// Meeting point of the NP producer waves of a workgroup (the workgroup barrier belongs to the tile hand-over, which
// the product waves take part in).  Every wave publishes the number of the meeting after its LDS traffic and waits
// until the others have published it too; both producers pass the same meetings in the same order.  The wait is
// bounded: a producer that never arrives (a programming error) ends in wrong results, not in a hung machine - and in
// a set bit in the call's status word (TileWs::status), which the host can read back, so that wrong results never
// go unnoticed.  The waiting waves look again as soon as the last look is back (no sleep in between: the meeting is
// on the tile's critical path, and a look is one LDS read for all four flags).
// The flags are reached through a pointer that says LDS.  Through a generic pointer these volatile accesses compile to
// flat instructions, and a flat read is only complete when every global read of the wave in flight is too (the next
// tile's points, depth texels): each look then cost a round trip to memory, some thousands of cycles per tile.
constexpr unsigned kStatusMeetingMissed = 1u;
typedef volatile int __attribute__((address_space(3))) * lds_flags;

template <int NP>
__device__ __forceinline__ void producers_meet(lds_flags flags, int w, int& seq, int lane, unsigned* status) {
  wave_sync();
  if constexpr (NP > 1) {
    ++seq;
    if (lane == 0) flags[w] = seq;
    static_assert(NP <= 4, "the four flags are read as one 16-byte vector");
    typedef int flags4 __attribute__((ext_vector_type(4)));
    typedef const volatile flags4 __attribute__((address_space(3))) * lds_flags4;
    bool all = false;
    for (int spins = 0; spins < (1 << 16) && !all; ++spins) {
      const flags4 f = *(lds_flags4)flags;   // one LDS round trip per look
      all = true;
#pragma unroll
      for (int o = 0; o < NP; ++o) all = all && (f[o] - seq >= 0);
    }
    if (!all && lane == 0) atomicOr(status, kStatusMeetingMissed);
    wave_sync();
  }
}

// What a producer wave knows about its pairs of one batch of views before the tests: projection, whether it lands in
// the image, the depth texel (requested, maybe still on its way) and, with a given selection, whether the view is kept.
template <int NP>
struct ProjectedBatch {
  Proj pj[kPBatch / 2 / NP];
  float dep[kPBatch / 2 / NP];
  bool fr[kPBatch / 2 / NP], kept[kPBatch / 2 / NP];
};

// First every projection and the request for its depth texel (and mask byte), nothing that waits for them: a wave has
// nobody to hide a read behind, so the reads of all its pairs are in flight together - and, for the first batch of a
// tile, while the wave still works on the tile before.
template <bool SEL, int NP>
__device__ __forceinline__ void project_batch(const FuseArgs& a, const ObjRange& ob, int blk, float3 pt, int vb0,
                                              lds_floats cam_lds, int w, int lane, ProjectedBatch<NP>& f) {
  constexpr int kTrips = kPBatch / 2 / NP;
  const int p = lane & 31, h = lane >> 5;
  const int nvb = min(kPBatch, ob.n_views - vb0);
  const int li0 = blk * kTilePts;
  const long long ip = ob.pt_begin + li0 + (li0 + p < ob.n_pts ? p : 0);
#pragma unroll
  for (int j = 0; j < kTrips; ++j) {
    const int it = w + NP * j;
    f.dep[j] = 1.0f;
    f.fr[j] = false;
    f.kept[j] = true;
    f.pj[j] = Proj{0.0f, 0.0f, 0.0f};
    if (2 * it >= nvb) continue;   // uniform
    const int vl = min(2 * it + h, nvb - 1);
    const int v = ob.view_begin + vb0 + vl;
    // the camera rows come from the LDS copy, through a pointer that says so: a generic read would wait for every
    // read in flight, the depth texels of the trips before included
    f.pj[j] = project(cam_lds + (vb0 + vl) * 16, pt.x, pt.y, pt.z);
    f.fr[j] = in_frustum(a.vis, f.pj[j]);
    if (a.vis.depth) f.dep[j] = a.vis.depth[(long long)v * a.vis.H * a.vis.W + (f.fr[j] ? depth_texel(a.vis, f.pj[j]) : 0)];
    if constexpr (SEL) f.kept[j] = view_kept(a, ip, vb0 + vl);
  }
}

// Builds tile `blk` of object `ob` into `stage` (room for `k_stage` k-steps) and `slot`.  pt: the lane's point; pre:
// the projected first batch of views (project_batch).  Called by all 64 lanes of
// each of the NP producer waves (w = 0 .. NP - 1), which share the views of the tile: wave w takes the trips
// it = w, w + NP, ... (two views per trip, one per half wave).  cam_lds: the object's camera rows in LDS.
template <int DT, bool SEL, int NP>
__device__ __forceinline__ void produce_tile(const FuseArgs& a, const ObjRange& ob, int blk,
                                             float3 pt, ProjectedBatch<NP>& pre, char* stage, int k_stage, int& dirty,
                                             TileSlot* slot, ProducerScratch* sc, lds_floats cam_lds, lds_flags flags,
                                             unsigned* status, int w, int& seq, int lane) {
  constexpr int kTrips = kPBatch / 2 / NP;   // trips of one wave per batch of views
  const int p = lane & 31, h = lane >> 5;
  const int Hf = a.feat.Hf, Wf = a.feat.Wf;
  const uint32_t row_bytes = (uint32_t)a.feat.D * 2u;
  const int li0 = blk * kTilePts;
  const bool p_valid = li0 + p < ob.n_pts;
  TileStep* st = reinterpret_cast<TileStep*>(stage);
  int used = 0, cnt = 0;
  bool exhausted = false;

  // zero weights, shared by the waves: complete for everybody at the first meeting, before any weight lands.  Only
  // the k-steps that the buffer's last tile wrote (`dirty` of them; all of the buffer the first time) can hold
  // anything but zeros.
  for (int q = w * kWave + lane; q < dirty * 128; q += NP * kWave)
    reinterpret_cast<u32x4*>(reinterpret_cast<char*>(&st[q >> 7]) + 64)[q & 127] = u32x4{0u, 0u, 0u, 0u};

  for (int vb0 = 0; vb0 < ob.n_views; vb0 += kPBatch) {
    const int nvb = min(kPBatch, ob.n_views - vb0);
    if (vb0 > 0) producers_meet<NP>(flags, w, seq, lane, status);   // the previous batch is done with the tables
    // the maps of this wave's views (view 2 it + h of trip it): 32 words each
#pragma unroll
    for (int j = 0; j < kTrips; ++j) {
      const int it = w + NP * j;
      reinterpret_cast<u32x4*>(&sc->bits[2 * it][0])[lane & 15] = u32x4{0u, 0u, 0u, 0u};   // 16 lanes x 16 bytes = two views
    }
    wave_sync();

    // ---- A: project and test; bounding box of the touched cells per view.  The projections and the requests for the
    // depth texels of the first batch were made a tile ago (project_batch); later batches make them here.
    PairRec pr[kTrips];
    if (vb0 > 0) project_batch<SEL, NP>(a, ob, blk, pt, vb0, cam_lds, w, lane, pre);
    Proj (&pj)[kTrips] = pre.pj;
    float (&dep)[kTrips] = pre.dep;
    bool (&fr)[kTrips] = pre.fr, (&kept)[kTrips] = pre.kept;
#pragma unroll
    for (int j = 0; j < kTrips; ++j) {
      const int it = w + NP * j;
      pr[j].xy = -1;
      pr[j].ax = pr[j].ay = 0.0f;
      if (2 * it >= nvb) continue;   // uniform
      const int vl = 2 * it + h;
      const bool seen = vl < nvb && p_valid && fr[j] && kept[j] && (a.vis.frustum_only || passes_depth(a.vis, pj[j], dep[j]));
      s16x2 lo2 = {0x7fff, 0x7fff}, hi2 = {-1, -1};
      if (seen) {
        const Tap tx = tap_axis(pj[j].u, a.feat.pitch_x, Wf), ty = tap_axis(pj[j].v, a.feat.pitch_y, Hf);
        pr[j].ax = tx.a;
        pr[j].ay = ty.a;
        pr[j].xy = (ty.i0 << 16) | tx.i0;
        lo2 = s16x2{(short)tx.i0, (short)ty.i0};
        hi2 = s16x2{(short)tx.i1, (short)ty.i1};
        ++cnt;
      }
      const unsigned long long seen_mask = __ballot(seen);
      lo2 = half_wave_reduce<true>(lo2);
      hi2 = half_wave_reduce<false>(hi2);
      if (p == kTilePts - 1 && vl < nvb) {
        const bool any = hi2[0] >= 0;
        const int ww = hi2[0] - lo2[0] + 1, wh = hi2[1] - lo2[1] + 1;
        sc->win[vl][0] = lo2[0];
        sc->win[vl][1] = lo2[1];
        sc->mode[vl] = !any ? 0 : (ww <= kWinSide && wh <= kWinSide ? 1 : 2);
        sc->vmask[vl] = (uint32_t)(seen_mask >> (lane & 32));
      }
    }
    wave_sync();

    // ---- B: mark the touched cells of this wave's views that use a map
#pragma unroll
    for (int j = 0; j < kTrips; ++j) {
      if (pr[j].xy < 0) continue;
      const int vl = 2 * (w + NP * j) + h;
      if (sc->mode[vl] != 1) continue;
      const int x0 = pr[j].xy & 0xffff, y0 = pr[j].xy >> 16;
      const int bit = (y0 - sc->win[vl][1]) * kWinSide + (x0 - sc->win[vl][0]);
      const bool has_x1 = x0 + 1 < Wf, has_y1 = y0 + 1 < Hf;
      atomicOr(&sc->bits[vl][bit >> 5], 1u << (bit & 31));
      if (has_x1) atomicOr(&sc->bits[vl][(bit + 1) >> 5], 1u << ((bit + 1) & 31));
      if (has_y1) atomicOr(&sc->bits[vl][(bit + kWinSide) >> 5], 1u << ((bit + kWinSide) & 31));
      if (has_x1 && has_y1) atomicOr(&sc->bits[vl][(bit + kWinSide + 1) >> 5], 1u << ((bit + kWinSide + 1) & 31));
    }
    producers_meet<NP>(flags, w, seq, lane, status);   // the maps, boxes and masks of all views are complete

    // the mask of Eq. 1 for this batch of views goes out with the tile: a product wave writes it to memory (a store
    // of a producer would hold up its next wait for a read: one counter covers both)
    if (w == 0 && a.out_vis && lane < nvb) slot->vmask[vb0 + lane] = sc->vmask[lane];
    {   // list length of every view, exclusive scan over the views: every producer wave does it (same values).
        // lane = (view, quarter of the map's rows): set bits before each row within the quarter, then the quarters'
        // totals through lane exchanges
      static_assert(kPBatch == 16 && kWinSide == 32, "lane = 16 views x 4 quarters of 8 rows");
      const int v = lane & 15, qd = lane >> 4;
      const bool map = v < nvb && sc->mode[v] == 1;
      int before[8], n = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        before[e] = n;
        n += map ? __popc(sc->bits[v][8 * qd + e]) : 0;
      }
      const int n0 = __shfl(n, v, kWave), n1 = __shfl(n, v + 16, kWave), n2 = __shfl(n, v + 32, kWave), n3 = __shfl(n, v + 48, kWave);
      const int off = (qd > 0 ? n0 : 0) + (qd > 1 ? n1 : 0) + (qd > 2 ? n2 : 0);
      if (map) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sc->wbase[v][8 * qd + e] = (uint16_t)(off + before[e]);
      }
      int total = n0 + n1 + n2 + n3;                                   // lanes 0 .. 15: the view's list length
      if (v < nvb && sc->mode[v] == 2) total = 4 * __popc(sc->vmask[v]);
      // running sum over the 16 views = over the first row of 16 lanes, with lane shifts inside the row (a lane without
      // a source adds 0): no trip through the LDS unit, which every exchange between arbitrary lanes would cost
      int inc = lane < kPBatch ? total : 0;
      inc = row_shift_add<0x111>(inc);   // row_shr:1
      inc = row_shift_add<0x112>(inc);   // row_shr:2
      inc = row_shift_add<0x114>(inc);   // row_shr:4
      inc = row_shift_add<0x118>(inc);   // row_shr:8
      if (lane < kPBatch) sc->base[lane] = inc - total;
      if (lane == kPBatch - 1) sc->base[kPBatch] = inc;
    }
    wave_sync();
    const int L = sc->base[kPBatch];
    const int nsteps = (L + kStepCells - 1) / kStepCells;
    if (used + nsteps > k_stage) {   // uniform, and the same in every producer wave
      exhausted = true;
      break;
    }
    TileStep* __restrict__ out = st + used;
    used += nsteps;

    // ---- C: the cells of the list, then the weights in the operand layout
    if (w == 0 && lane < nsteps * kStepCells - L) {   // entries that pad the last k-step point at a cell that exists
      const int idx = L + lane;
      out[idx >> 4].cell[idx & 15] = (uint32_t)((ob.view_begin + vb0) * Hf * Wf) * row_bytes;
    }
    {   // cells of the views with a map: lane = (view, rows of the map); the waves share the rows
      constexpr int kRows = 8 / NP;
      const int vl = lane >> 2, row0 = (kWinSide / NP) * w + kRows * (lane & 3);
      if (vl < nvb && sc->mode[vl] == 1) {
        const int cell0 = (ob.view_begin + vb0 + vl) * Hf + sc->win[vl][1], wx = sc->win[vl][0];
        for (int wd = row0; wd < row0 + kRows; ++wd) {
          uint32_t bits = sc->bits[vl][wd];
          int q = sc->base[vl] + sc->wbase[vl][wd];
          while (bits) {
            const int b = __builtin_ctz(bits);
            bits &= bits - 1;
            out[q >> 4].cell[q & 15] = (uint32_t)((cell0 + wd) * Wf + wx + b) * row_bytes;
            ++q;
          }
        }
      }
    }
    // list positions of the four cells of every pair first (LDS reads only), then the stores: with both in one loop
    // the reads of a pair would wait behind the stores of the pair before it
    int idx[kTrips][4];
#pragma unroll
    for (int j = 0; j < kTrips; ++j) {
#pragma unroll
      for (int k = 0; k < 4; ++k) idx[j][k] = 0;
      if (pr[j].xy < 0) continue;
      const int vl = 2 * (w + NP * j) + h;
      const int x0 = pr[j].xy & 0xffff, y0 = pr[j].xy >> 16;
      const bool has_x1 = x0 + 1 < Wf, has_y1 = y0 + 1 < Hf;
      const bool on[4] = {true, has_x1, has_y1, has_x1 && has_y1};
      if (sc->mode[vl] == 1) {
        const int bit = (y0 - sc->win[vl][1]) * kWinSide + (x0 - sc->win[vl][0]);
        const int bs[4] = {bit, bit + 1, bit + kWinSide, bit + kWinSide + 1};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int b = on[k] ? bs[k] : bit;
          idx[j][k] = sc->base[vl] + sc->wbase[vl][b >> 5] + __popc(sc->bits[vl][b >> 5] & ((1u << (b & 31)) - 1u));
        }
      } else {
        const int first = sc->base[vl] + 4 * __popc(sc->vmask[vl] & ((1u << p) - 1u));
#pragma unroll
        for (int k = 0; k < 4; ++k) idx[j][k] = -1 - (first + k);   // negative: a private entry, its cell is still to be written
      }
    }
    wave_sync();
#pragma unroll
    for (int j = 0; j < kTrips; ++j) {
      if (pr[j].xy < 0) continue;
      const int vl = 2 * (w + NP * j) + h;
      const int x0 = pr[j].xy & 0xffff, y0 = pr[j].xy >> 16;
      const float ax = pr[j].ax, ay = pr[j].ay;
      const bool has_x1 = x0 + 1 < Wf, has_y1 = y0 + 1 < Hf;
      const float wgt[4] = {(1.0f - ax) * (1.0f - ay), ax * (1.0f - ay), (1.0f - ax) * ay, ax * ay};
      const bool on[4] = {true, has_x1, has_y1, has_x1 && has_y1};
      if (idx[j][0] < 0) {
        const int cell0 = (ob.view_begin + vb0 + vl) * Hf;
        const int x1 = has_x1 ? x0 + 1 : x0, y1 = has_y1 ? y0 + 1 : y0;
        const int cx[4] = {x0, x1, x0, x1}, cy[4] = {y0, y0, y1, y1};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          idx[j][k] = -1 - idx[j][k];
          out[idx[j][k] >> 4].cell[idx[j][k] & 15] = (uint32_t)((cell0 + cy[k]) * Wf + cx[k]) * row_bytes;
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (on[k]) {
          uint16_t hi, lo;
          split_weight<DT>(wgt[k], hi, lo);
          const int c = idx[j][k] & 15;
          TileStep* stp = out + (idx[j][k] >> 4);
          reinterpret_cast<uint16_t*>(&stp->a_hi[(c >> 3) * kTilePts + p])[c & 7] = hi;
          reinterpret_cast<uint16_t*>(&stp->a_lo[(c >> 3) * kTilePts + p])[c & 7] = lo;
        }
      }
    }
  }

  const int mine = cnt + __shfl_xor(cnt, 32, kWave);   // views of this wave that see point lane % 32
  wave_sync();
  if (w == 0 && lane == 0) {
    slot->tile = blk;
    slot->nsteps = exhausted ? -1 : used;
    if (exhausted) atomicAdd(status + 1, 1u);   // second status word: tiles fused by the gather
  }
  if (lane < kTilePts) slot->cnt[w][lane] = mine;
  dirty = used;   // the same in every producer wave
  if (exhausted) gather_tile<DT>(a, ob, li0, w, NP, lane);   // writes the rows, the counts and the mask of the tile itself
}

// The scoring wave's part of a tile (Sec. 3.4.1): omega^T = G^T . W^T over the k-steps staged at `sb`, whose weight
// operand is exactly the B operand here; three partial products per k-step (hi * hi, hi * lo, lo * hi).  The rows of G
// of kScoreAhead k-steps are requested together (the wave has nobody to hide a read behind) and multiplied later.
// Accumulator element r of lane l is material 8 (r / 4) + 4 (l / 32) + r % 4 of point l % 32, before the point's factor.
constexpr int kScoreAhead = 8;

struct ScoreRows {
  uint32_t gv[kScoreAhead][8];
};

// What the scoring wave hands to a product wave for storing: a wave that stores to memory waits for the stores'
// acknowledgement before its next read comes back (one counter covers both), and the scoring wave lives on its reads.
struct __attribute__((aligned(16))) ScoreOut {
  float scores[kTilePts * kScoreTileM];   // [32][K]
  float prop[kTilePts * kScoreMaxP];      // [32][P]
  int label[kTilePts];
  int blk;                                // tile index within the object; -1: nothing to store
  int pad_[3];
};

// Requests G for those of the k-steps s0 .. s0 + kScoreAhead - 1 that exist (n staged ones).
__device__ __forceinline__ void request_rows(const char* sb, int n, int s0, const TileScoring& sc, uint32_t row_units, int lane,
                                             ScoreRows& rows) {
  const int pt = lane & 31, g = lane >> 5;
  const TileStep* st = reinterpret_cast<const TileStep*>(sb);
#pragma unroll
  for (int j = 0; j < kScoreAhead; ++j) {
    if (s0 + j >= n) break;   // uniform
    const TileStep* sj = st + s0 + j;
    const u32x4 c0 = *reinterpret_cast<const u32x4*>(&sj->cell[8 * g]);
    const u32x4 c1 = *reinterpret_cast<const u32x4*>(&sj->cell[8 * g + 4]);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      rows.gv[j][e] = sc.G[(long long)cell_index(e < 4 ? c0[e] : c1[e - 4], row_units) * sc.Kpad + pt];
  }
}

template <int DT>
__device__ __forceinline__ void multiply_rows(const char* sb, int n, int s0, const ScoreRows& rows, int lane, f32x16& acc) {
  const TileStep* st = reinterpret_cast<const TileStep*>(sb);
#pragma unroll
  for (int j = 0; j < kScoreAhead; ++j) {
    if (s0 + j < n) {
      const u32x4 w_hi = st[s0 + j].a_hi[lane], w_lo = st[s0 + j].a_lo[lane];
      u32x4 g_hi, g_lo;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        g_hi[q] = __builtin_amdgcn_perm(rows.gv[j][2 * q + 1], rows.gv[j][2 * q], 0x05040100u);
        g_lo[q] = __builtin_amdgcn_perm(rows.gv[j][2 * q + 1], rows.gv[j][2 * q], 0x07060302u);
      }
      acc = mma<DT>(g_hi, w_hi, acc);
      acc = mma<DT>(g_hi, w_lo, acc);
      acc = mma<DT>(g_lo, w_hi, acc);
    }
  }
}

// Stores what the scoring wave left in `o` (if anything): scores, properties and labels of the tile's points are
// contiguous in memory.  Called by all lanes of one wave.
__device__ __forceinline__ void store_scores(const ScoreOut& o, const TileScoring& sc, const ObjRange& ob, int lane) {
  const int blk = o.blk;
  if (blk < 0) return;
  const long long p0 = ob.pt_begin + (long long)blk * kTilePts;
  const int rows = min(kTilePts, ob.n_pts - blk * kTilePts);
  for (int q = lane; q < rows * sc.K; q += kWave) sc.scores[p0 * sc.K + q] = o.scores[q];
  if (sc.prop)
    for (int q = lane; q < rows * sc.P; q += kWave) sc.prop[p0 * sc.P + q] = o.prop[q];
  if (sc.label && lane < rows) sc.label[p0 + lane] = o.label[lane];
}

// S product waves and NP producer waves per workgroup; with SC one more wave, which scores the tiles (K <= 32).
template <int DT, int S, int H, int PF, bool SEL, int NP, bool SC>
__global__ __launch_bounds__(kWave* (S + NP + (SC ? 1 : 0))) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_tile_fused(FuseArgs fa, ProdArgs a, TileWs ws, int keep, ObjTable tab) {
  constexpr int kSpan = kHalf * H;
  constexpr int kStage = stage_steps_for<S * H / 2>();
  __shared__ __attribute__((aligned(16))) char s_steps[2][kStage * sizeof(TileStep)];
  __shared__ TileSlot s_slot[2];
  __shared__ __attribute__((aligned(16))) ProducerScratch s_sc;
  __shared__ float s_ss[2][S][kTilePts];
  __shared__ __attribute__((aligned(16))) float s_cam[kCamRows][16];   // the object's camera rows, for the producers
  __shared__ int s_plan[4];      // tickets of the workgroup's tiles, k-th tile in slot k & 3
  __shared__ __attribute__((aligned(16))) int s_flags[kMaxProducers];   // meeting numbers of the producer waves
  __shared__ float s_ys[SC ? kScoreTileM * kScoreMaxP : 1];   // the property table y[K][P]
  __shared__ ScoreOut s_out[SC ? 2 : 1];                        // scores of the tile before the last, on their way to memory

  const ObjRange ob = tab.o[blockIdx.y];
  const int nblk = (ob.n_pts + kTilePts - 1) / kTilePts;
  const int groups = min(nblk, (int)gridDim.x);
  if ((int)blockIdx.x >= groups) return;
  const int xcd = blockIdx.x % kXcd;
  const XcdTiles mine(nblk, xcd);
  const int len = mine.len;
  auto tile_at = [&](int t) { return mine.at(t); };
  unsigned* __restrict__ ctr = a.counters + blockIdx.y * kXcd + xcd;

  const int tid = threadIdx.x, lane = tid % kWave;
  // Wave index: the product waves come first, then the scoring wave if there is one, then the NP producers (waves go
  // to the four SIMDs in turn: every producer then shares its SIMD with a wave that leaves the vector ALU mostly alone).
  const int span = __builtin_amdgcn_readfirstlane(tid / kWave);
  constexpr int kFirstProducer = S + (SC ? 1 : 0);
  const bool producer = span >= kFirstProducer;
  const lds_floats cam_lds = (lds_floats)&s_cam[0][0];   // the launch code takes this kernel for up to kCamRows views
  const int m = lane & 31, g = lane >> 5;
  const int D = a.D;
  const uint32_t lane_off = (uint32_t)(span * kSpan + 4 * m) * 2u;

  if (producer) {
    // With eight waves in the workgroup every producer shares its SIMD with a product wave, and the tile waits for the
    // producers: they go first where both are ready (measured on 1024 channels with 24 views: 12 % faster; with seven
    // waves it does not pay).
    if constexpr (S + NP >= 8) __builtin_amdgcn_s_setprio(1);
    const int w = span - kFirstProducer;
    int seq = 0;
    // The first producer wave takes the tickets (the counters are zeroed by the launch that precedes this kernel) and
    // publishes them in s_plan, slot k & 3 for the k-th tile of the workgroup, two tiles ahead of the one being built:
    // at the top of a trip every producer knows the tile it builds now and the one after it.  Values of len or more
    // mean that the XCD's range is used up.
    auto ticket = [&]() {
      int t = 0;
      if (lane == 0) t = (int)atomicAdd(ctr, 1u);
      return t;
    };
    int t_raw = 0;   // the ticket of tile k + 3 while tile k + 1 is built (lane 0 of the first producer)
    if (w == 0) {
      for (int q = lane; q < ob.n_views * 16; q += kWave) s_cam[q >> 4][q & 15] = fa.vis.cam[(long long)ob.view_begin * 16 + q];
      const int t0 = ticket(), t1 = ticket(), t2 = ticket();
      t_raw = ticket();
      if (lane == 0) {
        s_plan[0] = t0;
        s_plan[1] = t1;
        s_plan[2] = t2;
        for (int o = 0; o < kMaxProducers; ++o) s_flags[o] = 0;
      }
    }
    __syncthreads();   // camera rows, the first plans and the meeting flags are in LDS
    const int last_tile = nblk - 1;
    // a plan past the end reads (and projects) a tile that exists; it is never built
    auto tile_of = [&](int t) { return min(tile_at(t), last_tile); };
    ProjectedBatch<NP> pre;
    int dirty0 = kStage, dirty1 = kStage;   // k-steps of each stage buffer that may hold non-zero weights
    float3 pt;   // the lane's point of the tile that the next trip builds
    {
      const int t0 = s_plan[0], t1 = s_plan[1];
      const float3 pt0 = tile_point(fa, ob, tile_of(t0), lane);
      const float3 pt1 = tile_point(fa, ob, tile_of(t1), lane);
      project_batch<SEL, NP>(fa, ob, tile_of(t0), pt0, 0, cam_lds, w, lane, pre);
      if (t0 < len) {
        produce_tile<DT, SEL, NP>(fa, ob, tile_at(t0), pt0, pre, s_steps[0], kStage, dirty0, &s_slot[0], &s_sc, cam_lds,
                                  (lds_flags)&s_flags[0], ws.status, w, seq, lane);
      } else if (w == 0 && lane == 0) {
        s_slot[0].tile = -1;
        s_slot[0].nsteps = 0;
      }
      project_batch<SEL, NP>(fa, ob, tile_of(t1), pt1, 0, cam_lds, w, lane, pre);
      pt = pt1;
    }
    __syncthreads();
    // Producers and product waves run loops with the same number of barriers: one trip per tile, ended by the barrier
    // after which the buffers change hands.  All leave when the slot they look at says that there is no further tile
    // (written before the last barrier, so every wave of the workgroup sees the same value).
    int buf = 0, k = 1;   // the trip builds the k-th tile of the workgroup
    while (s_slot[buf].tile >= 0) {
      const int t = s_plan[k & 3], tn = s_plan[(k + 1) & 3];
      const float3 pt_next = tile_point(fa, ob, tile_of(tn), lane);   // requested now, looked at after this tile is built
      if (t < len) {
        produce_tile<DT, SEL, NP>(fa, ob, tile_at(t), pt, pre, s_steps[buf ^ 1], kStage, buf ? dirty0 : dirty1, &s_slot[buf ^ 1], &s_sc, cam_lds,
                                  (lds_flags)&s_flags[0], ws.status, w, seq, lane);
      } else if (w == 0 && lane == 0) {
        s_slot[buf ^ 1].tile = -1;
        s_slot[buf ^ 1].nsteps = 0;
      }
      pt = pt_next;
      project_batch<SEL, NP>(fa, ob, tile_of(tn), pt, 0, cam_lds, w, lane, pre);   // its depth texels arrive during the barrier
      if (w == 0) {   // the plan of tile k + 2: its slot (k + 2) & 3 held tile k - 2, which nobody looks at any more
        const int t3 = __builtin_amdgcn_readfirstlane(t_raw);
        if (lane == 0) s_plan[(k + 2) & 3] = t3;
        if (t3 < len) t_raw = ticket();
      }
      __syncthreads();
      buf ^= 1;
      ++k;
    }
    return;
  }
  if constexpr (SC) {
    if (span == S) {
      // The scoring wave follows the product waves through the tiles, one barrier behind.  During a tile it multiplies
      // the staged weights with G.  After the tile's barrier the product waves' sums of squares are in LDS: the factor
      // of every point follows as in the product waves, and the scores, labels and properties of the tile go to LDS
      // (a product wave stores them during the next tile) while the rows of G for the next tile are on their way.
      const TileScoring& sc = fa.scoring;
      constexpr uint32_t row_units = S * H / 2;   // D / 256
      if (sc.prop)
        for (int t = lane; t < sc.K * sc.P; t += kWave) s_ys[t] = sc.y[t];
      if (lane == 0) s_out[0].blk = s_out[1].blk = -1;
      __syncthreads();
      __syncthreads();
      int buf = 0;
      int blk_prev = -1, n_prev = 0, cnt_prev = 0;   // the tile whose products are in acc
      f32x16 acc[1];
      while (true) {
        const int blk = s_slot[buf].tile;
        const int n = blk >= 0 ? s_slot[buf].nsteps : 0;
        int my_cnt = 0;
#pragma unroll
        for (int o = 0; o < NP; ++o) my_cnt += s_slot[buf].cnt[o][m];
        ScoreRows rows;
        if (n > 0) request_rows(s_steps[buf], n, 0, sc, row_units, lane, rows);

        if (blk_prev >= 0) {   // the tile before: its sums are in the other half of s_ss
          const int li = blk_prev * kTilePts + m;
          const bool valid = li < ob.n_pts;
          const long long ip = ob.pt_begin + (valid ? li : ob.n_pts - 1);
          // (a tile that the producers fused themselves, n_prev < 0, has its scores already: gather_tile)
          const float inv = cnt_prev > 0 ? 1.0f / (float)cnt_prev : 0.0f;
          float tot = 0.0f;
#pragma unroll
          for (int wv = 0; wv < S; ++wv) tot += s_ss[buf ^ 1][wv][m];
          const float normed = inv / fmaxf(sqrtf(tot) * inv, a.norm_eps);
          const float factor = a.mean_only ? inv : normed;
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[0][r] *= factor;
          if (blk >= 0) {   // a product wave stores the results during the next tile
            ScoreOut& o = s_out[buf ^ 1];
            if (valid && n_prev >= 0)
              finish_scores<1>(acc, (long long)m, g, sc.K, sc.P, sc.inv_T, s_ys, o.scores, sc.prop ? o.prop : nullptr,
                               sc.label ? o.label : nullptr, sc.unseen_zero != 0);
            if (lane == 0) o.blk = n_prev >= 0 ? blk_prev : -1;
          } else if (valid && n_prev >= 0) {   // the workgroup's last tile: nobody is left to hand it to
            finish_scores<1>(acc, ip, g, sc.K, sc.P, sc.inv_T, s_ys, sc.scores, sc.prop, sc.label, sc.unseen_zero != 0);
          }
        }
        if (blk < 0) break;

#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] = 0.0f;
        for (int s0 = 0; s0 < n; s0 += kScoreAhead) {
          if (s0 > 0) request_rows(s_steps[buf], n, s0, sc, row_units, lane, rows);
          multiply_rows<DT>(s_steps[buf], n, s0, rows, lane, acc[0]);
        }
        __syncthreads();
        blk_prev = blk;
        n_prev = n;
        cnt_prev = my_cnt;
        buf ^= 1;
      }
      return;
    }
  }
  __syncthreads();
  __syncthreads();

  StepA wa[2];
  StepC wc;
  StepQ<H> rq[PF];
  int buf = 0;
  if (s_slot[0].tile >= 0)
    open_tile<H, PF>(s_steps[0], min(max(s_slot[0].nsteps, 0), kStage), a.feat, lane_off, lane, g, wa, rq);

  while (true) {
    const int blk = s_slot[buf].tile;   // uniform over the workgroup: written before the last barrier
    if (blk < 0) break;
    const int n = s_slot[buf].nsteps;
    int my_cnt = 0;                      // views that see point (lane % 32) of this tile
#pragma unroll
    for (int o = 0; o < NP; ++o) my_cnt += s_slot[buf].cnt[o][m];
    f32x16 acc[4 * H];
#pragma unroll
    for (int t = 0; t < 4 * H; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

    const char* sb = s_steps[buf];
    {
      const int cnt = max(n, 0), l0 = cnt - 1;
      int s = 0;
      for (; s + PF <= cnt; s += PF) {
#pragma unroll
        for (int j = 0; j < PF; ++j) {
          lds_c(sb, min(s + j + PF, l0), g, wc);
          lds_a(sb, min(s + j + 1, l0), lane, wa[(j + 1) & 1]);
          mma_step<DT, H>(wa[j & 1], rq[j], acc);
          __builtin_amdgcn_sched_barrier(0);
          load_q(a.feat, wc, lane_off, rq[j]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int j = 0; j < PF - 1; ++j) {
        if (s + j < cnt) {
          lds_a(sb, min(s + j + 1, l0), lane, wa[(j + 1) & 1]);
          mma_step<DT, H>(wa[j & 1], rq[j], acc);
        }
      }
    }

    // What goes to memory besides the fused rows.  After the products, not before: the memory counter is in order
    // and covers stores as well, so a store issued ahead of the first product (behind a condition, which makes the
    // compiler count it as possibly absent) would have to be acknowledged before the cell rows requested earlier count
    // as arrived - one store round trip per tile on the critical path.
    if (n >= 0 && span == 0 && tid < kTilePts && fa.out_count && blk * kTilePts + tid < ob.n_pts)
      fa.out_count[ob.pt_begin + blk * kTilePts + tid] = my_cnt;
    if constexpr (SC) {   // what the scoring wave finished during the last tile (the tile before that one)
      if (span == (S > 1 ? 1 : 0)) store_scores(s_out[buf], fa.scoring, ob, lane);
    }
    if (keep && tid == 0) ws.hdr[ob.tile_begin + blk].nsteps = n;   // the scoring kernel reads the header from memory
    if (fa.out_vis && lane < kTilePts && blk * kTilePts + lane < ob.n_pts) {
      // The visibility mask (Eq. 1) of the tile, as aura_project_visibility writes it: lane = point, and the product
      // waves share the views, eight at a time (eight bytes of the point's row).  A tile that the producers fused
      // themselves has its mask already, up to the columns beyond the object's views.
      uint8_t* __restrict__ vrow = fa.out_vis + (ob.pt_begin + blk * kTilePts + lane) * fa.vis_pitch;
      const uint32_t* vm = s_slot[buf].vmask;
      if (n >= 0) {
        const bool pairs = (fa.vis_pitch & 7) == 0 && (reinterpret_cast<uintptr_t>(fa.out_vis) & 7) == 0;
        const bool words = (fa.vis_pitch & 3) == 0 && (reinterpret_cast<uintptr_t>(fa.out_vis) & 3) == 0;
        // who takes the first eight views, the next eight, ...: the last wave, the first, then the others, with the
        // second wave (which stores the scores where the workgroup has a scoring wave) at the end
        const int turn = S <= 2 ? span : (span == S - 1 ? 0 : (span == 0 ? 1 : (span == 1 ? S - 1 : span)));
        for (int v0 = 8 * turn; v0 < ob.n_views; v0 += 8 * S) {
          uint32_t wd[2] = {0u, 0u};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (v0 + e < ob.n_views) wd[e >> 2] |= ((vm[v0 + e] >> lane) & 1u) << (8 * (e & 3));
          if (pairs && v0 + 8 <= ob.n_views) {
            *reinterpret_cast<u32x2*>(vrow + v0) = u32x2{wd[0], wd[1]};
          } else {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
              if (words && v0 + 4 * q + 4 <= ob.n_views) {
                *reinterpret_cast<uint32_t*>(vrow + v0 + 4 * q) = wd[q];
              } else {
                for (int e = 0; e < 4 && v0 + 4 * q + e < ob.n_views; ++e) vrow[v0 + 4 * q + e] = (uint8_t)((wd[q] >> (8 * e)) & 1u);
              }
            }
          }
        }
      }
      if (span == S - 1)
        for (int j = ob.n_views; j < fa.vis_pitch; ++j) vrow[j] = 0;
    }
    if (keep && n > 0) {
      // The scoring kernel wants the k-steps in memory: the product waves, which have issue slots to spare, copy the
      // staged tile out (the producers do not: their vector ALU work is what the tile waits for).
      u32x4* __restrict__ dst = reinterpret_cast<u32x4*>(ws.steps + (long long)(ob.tile_begin + blk) * ws.quota);
      const u32x4* src = reinterpret_cast<const u32x4*>(sb);
      for (int q = span * kWave + lane; q < n * (int)(sizeof(TileStep) / 16); q += S * kWave) dst[q] = src[q];
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 8 * (r >> 2) + 4 * g + (r & 3);
      float ss = 0.0f;
#pragma unroll
      for (int t = 0; t < 4 * H; ++t) ss = __builtin_fmaf(acc[t][r], acc[t][r], ss);
      ss = half_wave_sum(ss);
      if (m == 31) s_ss[buf][span][row] = ss;
    }
    __syncthreads();   // the one barrier of a tile: the sums are in LDS, the producers have staged the next tile, and
                       // every product wave is done with this tile's buffer

    float factor;
    {
      const float inv = my_cnt > 0 ? 1.0f / (float)my_cnt : 0.0f;
      float tot = 0.0f;
#pragma unroll
      for (int wv = 0; wv < S; ++wv) tot += s_ss[buf][wv][m];
      const float normed = inv / fmaxf(sqrtf(tot) * inv, a.norm_eps);
      factor = a.mean_only ? inv : normed;
    }
    {
      const int rows_f = a.factor ? min(kTilePts, ob.n_pts - blk * kTilePts) : 0;
      const __amdgpu_buffer_rsrc_t fout = __builtin_amdgcn_make_buffer_rsrc(a.factor + (a.factor ? ob.pt_begin + blk * kTilePts : 0), 0,
                                                                            rows_f * 4, 0x00020000);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_int(factor), fout, tid < kTilePts ? 4 * tid : 0x7ffffff0, 0, 0);
    }
    {
      const int li0 = blk * kTilePts;
      float* obase = a.fused ? a.fused + (ob.pt_begin + li0) * D + span * kSpan : nullptr;
      uint32_t row_bytes = (uint32_t)D * 4u;
      asm volatile("" : "+s"(row_bytes));
      const int rows = (n >= 0 && a.fused) ? min(kTilePts, ob.n_pts - li0) : 0;
      const __amdgpu_buffer_rsrc_t out = __builtin_amdgcn_make_buffer_rsrc(obase, 0, (int)(rows * row_bytes), 0x00020000);
      const uint32_t lane_out = (uint32_t)(4 * g) * row_bytes + (uint32_t)(4 * m) * 4u;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row0 = 8 * (r >> 2) + (r & 3);
        const float scale = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (row0 + 4 * g), __float_as_int(factor)));
#pragma unroll
        for (int h = 0; h < H; ++h) {
          const f32x4 v = {acc[4 * h][r] * scale, acc[4 * h + 1][r] * scale, acc[4 * h + 2][r] * scale, acc[4 * h + 3][r] * scale};
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), out,
                                                 (int)(lane_out + (uint32_t)row0 * row_bytes) + h * kHalf * 4, 0, /*streaming*/ 2);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    buf ^= 1;
    {
      const int nn = s_slot[buf].tile >= 0 ? min(max(s_slot[buf].nsteps, 0), kStage) : 0;
      open_tile<H, PF>(s_steps[buf], nn, a.feat, lane_off, lane, g, wa, rq);
    }
  }
  if constexpr (SC) {   // the tile before the workgroup's last one (the scoring wave stores the last one itself)
    if (span == (S > 1 ? 1 : 0)) store_scores(s_out[buf], fa.scoring, ob, lane);
  }
}

// Clears the ticket counters of a launch's objects (the prepare kernel does it on the two-kernel path).
__global__ void k_clear_counters(unsigned* counters, int n, unsigned* status) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) counters[i] = 0u;
  if (i == 0 && status) {
    status[0] = 0u;
    status[1] = 0u;
  }
}

// ------------------------------------------------------------------------------------ host

static long long tile_count_bound(long long N, int B) { return N / kTilePts + B; }

static int steps_quota(int B, int n_views) {
  // k-steps of storage per tile: two per view of an object, within [4, 32] (measured need on
  // spatially sorted points: 0.3 to 0.4 per view for coarse grids, up to 1 for pixel-sized cells)
  const long long per_obj = (n_views + B - 1) / B;
  return (int)(2 * per_obj < 4 ? 4 : (2 * per_obj > 32 ? 32 : 2 * per_obj));
}

static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t fuse_tile_workspace_bytes(long long N, int B, int n_views) {
  const size_t tiles = (size_t)tile_count_bound(N, B);
  return round256(tiles * sizeof(TileHdr)) + round256((size_t)B * 8 * sizeof(unsigned)) + 256 +
         tiles * (size_t)steps_quota(B, n_views) * sizeof(TileStep);
}

TileWs fuse_tile_workspace(void* workspace, long long N, int B, int n_views) {
  char* base = static_cast<char*>(workspace);
  TileWs ws;
  ws.hdr = reinterpret_cast<TileHdr*>(base);
  base += round256((size_t)tile_count_bound(N, B) * sizeof(TileHdr));
  ws.counters = reinterpret_cast<unsigned*>(base);
  base += round256((size_t)B * 8 * sizeof(unsigned));
  ws.status = reinterpret_cast<unsigned*>(base);
  base += 256;
  ws.steps = reinterpret_cast<TileStep*>(base);
  ws.quota = steps_quota(B, n_views);
  ws.obj_base = 0;
  return ws;
}

size_t fuse_tile_status_offset(long long N, int B) {
  return round256((size_t)tile_count_bound(N, B) * sizeof(TileHdr)) + round256((size_t)B * 8 * sizeof(unsigned));
}

bool fuse_tile_supported(int dtype, int D, int Hf, int Wf, long long feat_bytes) {
  // cell coordinates travel as 16-bit pairs and cell rows as 32-bit byte offsets inside the kernels
  return (dtype == 1 || dtype == 2) && Hf <= 32767 && Wf <= 32767 && D % 256 == 0 && D / 256 >= 1 && D / 256 <= 6 &&
         D / 256 != 5 && feat_bytes <= 0xffffffffll;
}

// How many producer waves the one-kernel form takes for this launch; 0: the two kernels.  The lists of (nearly) all
// tiles must fit the LDS buffer of kStage k-steps, and when the scoring kernel wants the k-steps in memory, the
// tile's share of the workspace as well.  Measured need on spatially sorted points: 0.3 to 0.4 k-steps per view for
// coarse grids, up to 1 for pixel-sized cells.  One producer wave keeps up with the product waves for a few views per
// object; beyond that four share the views of a tile and a compute unit holds one workgroup of at most eight waves
// (two per SIMD: a product wave needs about 250 registers).
static int one_kernel_producers(const FuseArgs& a, int k_stage, int quota, int views_per_obj, int product_waves) {
  const float per_view = (a.feat.pitch_x >= 4.0f && a.feat.pitch_y >= 4.0f) ? 0.5f : 1.0f;
  if (a.two_kernels || k_stage > quota || views_per_obj > kCamRows || (float)views_per_obj * per_view > (float)k_stage) return 0;
  if (views_per_obj <= kOneKernelViews) return 1;
  if (product_waves + 4 > 8) return 0;
  // (where the scoring kernel wants the k-steps in memory the product waves copy them out: measured 3 to 7 % faster than
  // the two kernels on 768 channels with 16 views and on 1024 channels with 24 views)
  return 4;
}

// Whether the one-kernel form of this launch can score its tiles itself: a scoring wave must fit the workgroup (at most
// three product waves beside the four producers) and one matrix-core tile must hold the materials.
static bool scoring_wave_fits(const FuseArgs& a, int producers, int product_waves) {
  // With one producer wave (two workgroups of up to four waves per compute unit) the scoring wave pays where no rows are
  // stored (the single-pass call: C5 2.63 -> 2.45 ms): with rows the call is bound by their stores either way, and the
  // separate scoring kernel keeps the fusion kernel shorter (C5 combined call 3.12 ms against 3.16 ms).
  const bool fits = (producers == 4 && product_waves + 4 + 1 <= 8) ||
                    (producers == 1 && product_waves + 1 + 1 <= 4 && a.fused == nullptr);
  return fits && a.out_factor && a.scoring.G && a.scoring.Kpad == kScoreTileM && !a.in_mask;
}

template <int DT, int S, int H, int PF>
static hipError_t launch_tile(const FuseArgs& a, const TileWs& ws, const ObjTable& tab, int n_obj, int max_pts,
                              hipStream_t stream, bool* scored) {
  const int max_tiles = (max_pts + kTilePts - 1) / kTilePts;
  ProdArgs pa{static_cast<const char*>(a.feat.feat), a.feat.D, ws.hdr, ws.steps, ws.counters + (size_t)ws.obj_base * kXcd,
              ws.quota, a.fused, a.out_factor, a.norm_eps, a.mean_only};
  int max_views = 0;
  for (int t = 0; t < n_obj; ++t) max_views = std::max(max_views, tab.o[t].n_views);
  const int np = one_kernel_producers(a, stage_steps_for<S * H / 2>(), ws.quota, max_views, S);
  if (np > 0) {
    // (the status word of the call is cleared along with the counters of its first launch)
    hipLaunchKernelGGL(k_clear_counters, dim3((n_obj * kXcd + 63) / 64), dim3(64), 0, stream, pa.counters, n_obj * kXcd,
                       ws.obj_base == 0 ? ws.status : nullptr);
    // with one producer wave two workgroups fit a compute unit, with four one; several objects in one launch share
    // the machine
    const int groups_max = np == 1 ? kFusedGroupsMax : kFusedGroupsMax / 2;
    const bool scoring = scoring_wave_fits(a, np, S);
    const int keep = a.out_factor != nullptr && !scoring;   // the scoring kernel follows and reads the k-steps
    // Several objects in one launch: many more workgroups per object than are resident at a time.  The workgroups of
    // an object share its tiles through the per-XCD tickets and are dispatched object after object, so the machine
    // works on a few objects at a time - their depth and feature maps stay in L2, where with eight workgroups per object
    // all 64 objects of a launch were in progress at once - and no workgroup is left with a fixed share of one object
    // while others have run out (64 objects of 100 000 points and 4 views: the workgroups' end times were spread over
    // the last quarter of the kernel; fusion call 2.79 -> 2.33 ms with 256 workgroups per object, the combined call,
    // whose workgroups also write the k-steps for the scoring kernel, 3.10 -> 2.94 ms with 64 and slower beyond).
    const int per_object = n_obj > 1 ? ((keep || scoring) ? 64 : 256) : 0;
    const int groups = std::max(kXcd, std::min(max_tiles, std::max((groups_max / n_obj + kXcd - 1) / kXcd * kXcd, per_object)));
    const dim3 grid(std::min(groups, max_tiles), n_obj), block(kWave * (S + np + (scoring ? 1 : 0)));
    const TimingRequest timed = take_timing_request();
    if (timed.start) (void)hipEventRecord(timed.start, stream);
    if (scoring) {
      pa.factor = nullptr;   // nobody reads the factors back
      if (np == 1) {
        if constexpr (S <= 2) hipLaunchKernelGGL((k_tile_fused<DT, S, H, PF, false, 1, true>), grid, block, 0, stream, a, pa, ws, keep, tab);
      } else {
        if constexpr (S <= 3) hipLaunchKernelGGL((k_tile_fused<DT, S, H, PF, false, 4, true>), grid, block, 0, stream, a, pa, ws, keep, tab);
      }
      if (scored) *scored = true;
    } else if (np == 1) {
      if (a.in_mask) hipLaunchKernelGGL((k_tile_fused<DT, S, H, PF, true, 1, false>), grid, block, 0, stream, a, pa, ws, keep, tab);
      else hipLaunchKernelGGL((k_tile_fused<DT, S, H, PF, false, 1, false>), grid, block, 0, stream, a, pa, ws, keep, tab);
    } else if constexpr (S + 4 <= 8) {
      if (a.in_mask) hipLaunchKernelGGL((k_tile_fused<DT, S, H, PF, true, 4, false>), grid, block, 0, stream, a, pa, ws, keep, tab);
      else hipLaunchKernelGGL((k_tile_fused<DT, S, H, PF, false, 4, false>), grid, block, 0, stream, a, pa, ws, keep, tab);
    }
    const hipError_t e = hipGetLastError();
    if (timed.stop) (void)hipEventRecord(timed.stop, stream);
    return e;
  }
  if (ws.obj_base == 0) {   // the status words of the call (the prepare kernel clears its objects' ticket counters itself)
    hipLaunchKernelGGL(k_clear_counters, dim3(1), dim3(64), 0, stream, pa.counters, 0, ws.status);
    const hipError_t ec = hipGetLastError();
    if (ec != hipSuccess) return ec;
  }
  const TimingRequest timed = take_timing_request();   // two kernels: the events go around the pair
  if (timed.start) (void)hipEventRecord(timed.start, stream);
  if (a.in_mask)
    hipLaunchKernelGGL((k_tile_prepare<DT, true>), dim3(max_tiles, n_obj), dim3(kPrepThreads), 0, stream, a, ws, tab);
  else
    hipLaunchKernelGGL((k_tile_prepare<DT, false>), dim3(max_tiles, n_obj), dim3(kPrepThreads), 0, stream, a, ws, tab);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // several objects in one launch share the machine: fewer workgroups per object
  const int groups = std::max(kXcd, std::min(max_tiles, (kProdGroupsMax / n_obj + kXcd - 1) / kXcd * kXcd));
  hipLaunchKernelGGL((k_tile_product<DT, S, H, PF>), dim3(std::min(groups, max_tiles), n_obj), dim3(kWave * S), 0, stream, pa, tab);
  e = hipGetLastError();
  if (timed.stop) (void)hipEventRecord(timed.stop, stream);
  return e;
}

hipError_t launch_fuse_tile(const FuseArgs& a, const TileWs& ws, const ObjTable& tab, int n_obj, int max_pts,
                            hipStream_t stream, bool* scored) {
  if (scored) *scored = false;
  // waves x pieces of 128 channels per wave x k-steps of rows requested ahead, for each supported D
#define AURA_TILE_CASE(d, s, h, pf)                                                           \
  case d:                                                                                     \
    return a.feat.dtype == 1 ? launch_tile<1, s, h, pf>(a, ws, tab, n_obj, max_pts, stream, scored)   \
                             : launch_tile<2, s, h, pf>(a, ws, tab, n_obj, max_pts, stream, scored)
  switch (a.feat.D) {
    AURA_TILE_CASE(256, 1, 2, 2);
    AURA_TILE_CASE(512, 2, 2, 2);
    AURA_TILE_CASE(768, 3, 2, 2);
    AURA_TILE_CASE(1024, 4, 2, 2);
    AURA_TILE_CASE(1536, 6, 2, 2);
    default: return hipErrorInvalidValue;
  }
#undef AURA_TILE_CASE
}

}  // namespace aura
