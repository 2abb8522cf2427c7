// aura_fuse_features, matrix-core path (Sec. 3.1 "Feature Aggregation", Eq. 2).
//
// Eq. 2 with bilinear sampling is a weighted sum of feature cells:
//     sum_v M_vis(x_i, v) F_v(pi(x_i, v)) = sum_c  w[i][c] * F[c],
// where c runs over (view, cell) pairs and w[i][c] is the bilinear weight of cell c for point i
// (zero unless the view sees the point and c is one of the four cells around the projection).
// For 32 spatially neighbouring points the cells with a non-zero weight fall, per view, inside a
// small window of the feature grid (a few cells), so the sum is a small dense product
//     [32 points x L cells] . [L cells x D channels]
// with L around one hundred.  The gather formulation reads every cell row once per point and view
// (4 D elements per pair) and spends its time widening and multiplying on the vector ALUs; the
// dense form reads each cell of the window once per 32 points and runs on the matrix cores, which
// take the stored 16-bit features as they are.
//
// One workgroup fuses 32 consecutive points; wave s of the workgroup owns channels
// [256 s, 256 s + 256).
//   A  every (point, view) pair is projected and tested (Eq. 1, the shared fp32 decision
//      functions); each view's window = bounding box of the cells touched by the points it sees.
//   B  the windows are laid end to end into a cell list; the weights are scattered into a
//      [32][L] matrix in LDS, split into two 16-bit terms (hi + lo) so that the product carries
//      about 16 mantissa bits of each weight.
//   C  per 16 cells: each lane reads 16 bytes (8 channels) of 8 cell rows straight from global
//      memory, regroups them into the 8 B-operands (one per channel phase t = channel mod 8),
//      and issues v_mfma_f32_32x32x16 with the hi and the lo weights.  Lists longer than the LDS
//      matrix are processed in chunks; more than 32 views per object in batches.
//   D  mean, L2 norm (half-wave reduction, then across the waves through LDS), streaming store.
//      Accumulator t, register r of lane l is point 8 (r/4) + 4 (l/32) + r%4, channel
//      256 s + 8 (l%32) + t: every lane stores 8 consecutive channels of a point.
//
// Weights of cells that only pad a window (no point taps them) are zero, so feature maps must be
// finite everywhere.  Points that are far apart (unsorted input) give large windows: the kernel
// stays correct but loses its advantage; the gather kernel can be forced with AURA_FUSE_GATHER.
#include "aura_device.hpp"
#include "fuse_args.hpp"
#include "launch.hpp"

namespace aura {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr int kTilePts = 32;      // points per workgroup (M of the MFMA tile)
constexpr int kViewBatch = 32;    // views handled per pass over the point tile
constexpr int kListMax = 128;     // cells per chunk of the weight matrix in LDS
constexpr int kListPad = kListMax + 8;   // row pitch: consecutive rows start 4 banks apart
constexpr int kSpan = 256;        // channels per wave: 32 lanes x 8 channels

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

template <int DT>
__device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c) {
  if constexpr (DT == 1)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Reads the 8 cell rows of k-step s for this lane: 16 bytes (8 channels) of each.
__device__ __forceinline__ void load_cells(const char* __restrict__ fbase, const int* s_cell, int s, int g, int D,
                                           u32x4 (&q)[8]) {
  const i32x4 ca = *reinterpret_cast<const i32x4*>(&s_cell[16 * s + 8 * g]);
  const i32x4 cb = *reinterpret_cast<const i32x4*>(&s_cell[16 * s + 8 * g + 4]);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int cell = e < 4 ? ca[e] : cb[e - 4];
    q[e] = *reinterpret_cast<const u32x4*>(fbase + (long long)cell * D * 2);
  }
}

// 16 matrix-core instructions of one k-step: operand t holds channel 8 m + t of the 8 cells.
template <int DT>
__device__ __forceinline__ void mma_step(const u32x4& ah, const u32x4& al, const u32x4 (&q)[8], f32x16 (&acc)[8]) {
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    u32x4 b;
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      // bytes 0..3 of the selector index the first cell's dword, 4..7 the second cell's
      const uint32_t lo = q[2 * e2][t >> 1], hi = q[2 * e2 + 1][t >> 1];
      b[e2] = __builtin_amdgcn_perm(hi, lo, (t & 1) ? 0x07060302u : 0x05040100u);
    }
    acc[t] = mma<DT>(ah, b, acc[t]);
    acc[t] = mma<DT>(al, b, acc[t]);
  }
}

// DT: 1 bf16, 2 fp16 feature maps.  S waves per workgroup, D == 256 * S.
template <int DT, int S>
__global__ __launch_bounds__(kWave* S) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_fuse_tile(FuseArgs a, ObjTable tab) {
  constexpr int T = kWave * S;
  constexpr int NIT = (kViewBatch + 2 * S - 1) / (2 * S);   // (point, view) pairs per thread and batch
  __shared__ int s_xy[kViewBatch][kTilePts];        // y0 << 16 | x0, or -1: not visible
  __shared__ float s_ax[kViewBatch][kTilePts];
  __shared__ float s_ay[kViewBatch][kTilePts];
  __shared__ int s_win[kViewBatch][4];              // xmin, ymin, width, height of the view's window
  __shared__ int s_base[kViewBatch + 1];            // first list index of each view's window
  __shared__ __attribute__((aligned(16))) int s_cell[kListMax];   // cell index (view, y, x flattened) per list entry
  __shared__ __attribute__((aligned(16))) uint16_t s_whi[kTilePts][kListPad];
  __shared__ __attribute__((aligned(16))) uint16_t s_wlo[kTilePts][kListPad];
  __shared__ float s_ss[S][kTilePts];
  __shared__ int s_cnt[kTilePts];
  __shared__ float s_scale[kTilePts];

  const ObjRange ob = tab.o[blockIdx.y];
  const int nblk = (ob.n_pts + kTilePts - 1) / kTilePts;
  if ((int)blockIdx.x >= nblk) return;
  const int blk = xcd_contiguous(blockIdx.x, nblk);
  const int tid = threadIdx.x, lane = tid % kWave, span = tid / kWave;
  const int D = a.feat.D, Hf = a.feat.Hf, Wf = a.feat.Wf;
  const int p = tid % kTilePts;          // point of this thread in phases A and B
  const int slot = tid / kTilePts;       // view slot of this thread in phases A and B
  const int li0 = blk * kTilePts;
  const bool p_valid = li0 + p < ob.n_pts;
  const long long ip = ob.pt_begin + li0 + (p_valid ? p : 0);
  const float px = a.xyz[3 * ip], py = a.xyz[3 * ip + 1], pz = a.xyz[3 * ip + 2];
  const int m = lane & 31, g = lane >> 5;
  const char* fbase = static_cast<const char*>(a.feat.feat) + ((long long)span * kSpan + 8 * m) * 2;

  f32x16 acc[8];
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

  if (tid < kTilePts) s_cnt[tid] = 0;

  for (int vb0 = 0; vb0 < ob.n_views; vb0 += kViewBatch) {
    const int nvb = min(kViewBatch, ob.n_views - vb0);
    __syncthreads();   // previous batch fully consumed (and s_cnt initialised)

    // ---- A: project and test.  All projections first and the depth reads unconditional (at a
    // clamped texel), so that the reads of all pairs of a thread are in flight together.
    Proj pr[NIT];
    float dep[NIT];
    bool fr[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int vl = min(it * 2 * S + slot, nvb - 1);
      const int v = ob.view_begin + vb0 + vl;
      pr[it] = project(a.vis.cam + (long long)v * 16, px, py, pz);
      fr[it] = in_frustum(a.vis, pr[it]);
      dep[it] = 1.0f;
      if (a.vis.depth) dep[it] = a.vis.depth[(long long)v * a.vis.H * a.vis.W + (fr[it] ? depth_texel(a.vis, pr[it]) : 0)];
    }
    int my_cnt = 0;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int vl = it * 2 * S + slot;
      int xy = -1;
      s16x2 lo2 = {0x7fff, 0x7fff}, hi2 = {-1, -1};   // (x, y) of the first / second cell, 16 bits each
      float ax = 0.0f, ay = 0.0f;
      const bool seen = vl < nvb && p_valid && fr[it] && (a.vis.frustum_only || passes_depth(a.vis, pr[it], dep[it]));
      if (seen) {
        const Tap tx = tap_axis(pr[it].u, a.feat.pitch_x, Wf), ty = tap_axis(pr[it].v, a.feat.pitch_y, Hf);
        ax = tx.a;
        ay = ty.a;
        xy = (ty.i0 << 16) | tx.i0;
        lo2 = s16x2{(short)tx.i0, (short)ty.i0};
        hi2 = s16x2{(short)tx.i1, (short)ty.i1};
        ++my_cnt;
      }
      // bounding box over the 32 points of this view (the 32 lanes of a half wave share vl)
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) {
        lo2 = __builtin_elementwise_min(lo2, __builtin_bit_cast(s16x2, __shfl_xor(__builtin_bit_cast(int, lo2), o, kWave)));
        hi2 = __builtin_elementwise_max(hi2, __builtin_bit_cast(s16x2, __shfl_xor(__builtin_bit_cast(int, hi2), o, kWave)));
      }
      const int bx0 = lo2[0], by0 = lo2[1], bx1 = hi2[0], by1 = hi2[1];
      if (vl < nvb) {
        s_xy[vl][p] = xy;
        s_ax[vl][p] = ax;
        s_ay[vl][p] = ay;
        if (p == 0) {
          const bool any = bx1 >= 0;
          s_win[vl][0] = any ? bx0 : 0;
          s_win[vl][1] = any ? by0 : 0;
          s_win[vl][2] = any ? bx1 - bx0 + 1 : 0;
          s_win[vl][3] = any ? by1 - by0 + 1 : 0;
        }
      }
    }
    if (my_cnt) atomicAdd(&s_cnt[p], my_cnt);
    __syncthreads();
    if (tid < kWave) {   // exclusive scan of the window sizes by the first wave
      const int sz = lane < nvb ? s_win[lane][2] * s_win[lane][3] : 0;
      int inc = sz;
#pragma unroll
      for (int o = 1; o < kViewBatch; o <<= 1) {
        const int up = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += up;
      }
      if (lane < nvb) s_base[lane] = inc - sz;
      if (lane == nvb - 1) s_base[nvb] = inc;
    }
    __syncthreads();
    const int L = s_base[nvb];

    // ---- B + C: chunks of the cell list
    for (int c0 = 0; c0 < L; c0 += kListMax) {
      const int Lc = min(kListMax, L - c0);
      const int ksteps = (Lc + 15) / 16;
      if (c0 > 0) __syncthreads();   // the previous chunk's operands have been read
      // zero the weight matrix (16 bytes per store)
      for (int q = tid; q < kTilePts * ksteps * 2; q += T) {
        const int row = q / (ksteps * 2), col = (q % (ksteps * 2)) * 8;
        const u32x4 z = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(&s_whi[row][col]) = z;
        *reinterpret_cast<u32x4*>(&s_wlo[row][col]) = z;
      }
      // cell index of every list entry of the chunk: each view's window is enumerated row by row;
      // the entries that pad the last k-step point at a cell that exists (their weights are zero)
      {
        const int vl = tid % kViewBatch;
        if (vl < nvb) {
          const int wx = s_win[vl][0], wy = s_win[vl][1], ww = s_win[vl][2], n = ww * s_win[vl][3];
          const int base = s_base[vl] - c0, cell0 = (ob.view_begin + vb0 + vl) * Hf;
          for (int local = tid / kViewBatch; local < n; local += T / kViewBatch) {
            const int q = base + local;
            if (q >= 0 && q < Lc) s_cell[q] = (cell0 + wy + local / ww) * Wf + wx + local % ww;
          }
        }
        if (tid >= Lc && tid < ksteps * 16) s_cell[tid] = (ob.view_begin + vb0) * Hf * Wf;
      }
      __syncthreads();
      // scatter the bilinear weights of every visible (point, view) pair
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int vl = it * 2 * S + slot;
        if (vl >= nvb) continue;
        const int xy = s_xy[vl][p];
        if (xy < 0) continue;
        const int x0 = xy & 0xffff, y0 = xy >> 16;
        const float ax = s_ax[vl][p], ay = s_ay[vl][p];
        const int wx = s_win[vl][0], wy = s_win[vl][1], ww = s_win[vl][2];
        const int i00 = s_base[vl] + (y0 - wy) * ww + (x0 - wx) - c0;
        const bool has_x1 = x0 + 1 < Wf, has_y1 = y0 + 1 < Hf;   // at the border the second cell has weight 0
        const float wgt[4] = {(1.0f - ax) * (1.0f - ay), ax * (1.0f - ay), (1.0f - ax) * ay, ax * ay};
        const int idx[4] = {i00, i00 + 1, i00 + ww, i00 + ww + 1};
        const bool on[4] = {true, has_x1, has_y1, has_x1 && has_y1};
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
      // ---- C: matrix-core product for this wave's 256 channels; the cell rows of the next k-step
      // are requested before the products of the current one are issued
      {
        u32x4 q0[8], q1[8];
        load_cells(fbase, s_cell, 0, g, D, q0);
        for (int s = 0; s < ksteps; s += 2) {
          if (s + 1 < ksteps) load_cells(fbase, s_cell, s + 1, g, D, q1);
          {
            const u32x4 ah = *reinterpret_cast<const u32x4*>(&s_whi[m][16 * s + 8 * g]);
            const u32x4 al = *reinterpret_cast<const u32x4*>(&s_wlo[m][16 * s + 8 * g]);
            mma_step<DT>(ah, al, q0, acc);
          }
          if (s + 1 < ksteps) {
            if (s + 2 < ksteps) load_cells(fbase, s_cell, s + 2, g, D, q0);
            const u32x4 ah = *reinterpret_cast<const u32x4*>(&s_whi[m][16 * (s + 1) + 8 * g]);
            const u32x4 al = *reinterpret_cast<const u32x4*>(&s_wlo[m][16 * (s + 1) + 8 * g]);
            mma_step<DT>(ah, al, q1, acc);
          }
        }
      }
    }
  }

  // ---- D: mean, L2 norm, store.  One factor per point, inv_count / max(norm of the mean, eps),
  // is computed once and applied to the raw sums.
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = 8 * (r >> 2) + 4 * g + (r & 3);
    float ss = 0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t) ss = __builtin_fmaf(acc[t][r], acc[t][r], ss);
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) ss += __shfl_xor(ss, o, kWave);
    if (m == 0) s_ss[span][row] = ss;
  }
  __syncthreads();
  if (tid < kTilePts) {
    const int c = s_cnt[tid];
    const float inv = c > 0 ? 1.0f / (float)c : 0.0f;
    float f = inv;
    if (!a.mean_only) {
      float tot = 0.0f;
#pragma unroll
      for (int w = 0; w < S; ++w) tot += s_ss[w][tid];
      f = inv / fmaxf(sqrtf(tot) * inv, a.norm_eps);
    }
    s_scale[tid] = f;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = 8 * (r >> 2) + 4 * g + (r & 3);
    if (li0 + row >= ob.n_pts) continue;
    const float scale = s_scale[row];
    float* o = a.fused + (ob.pt_begin + li0 + row) * D + span * kSpan + 8 * m;
    const f32x4 v0 = {acc[0][r] * scale, acc[1][r] * scale, acc[2][r] * scale, acc[3][r] * scale};
    const f32x4 v1 = {acc[4][r] * scale, acc[5][r] * scale, acc[6][r] * scale, acc[7][r] * scale};
    __builtin_nontemporal_store(v0, reinterpret_cast<f32x4*>(o));
    __builtin_nontemporal_store(v1, reinterpret_cast<f32x4*>(o + 4));
  }
  if (a.out_count && tid < kTilePts && li0 + tid < ob.n_pts) a.out_count[ob.pt_begin + li0 + tid] = s_cnt[tid];
}

template <int DT, int S>
static hipError_t launch_tile(const FuseArgs& a, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream) {
  dim3 grid((max_pts + kTilePts - 1) / kTilePts, n_obj), block(kWave * S);
  hipLaunchKernelGGL((k_fuse_tile<DT, S>), grid, block, 0, stream, a, tab);
  return hipGetLastError();
}

bool fuse_tile_supported(int dtype, int D, int Hf, int Wf) {
  // cell coordinates travel as 16-bit pairs inside the kernel
  return (dtype == 1 || dtype == 2) && Hf <= 32767 && Wf <= 32767 && D % kSpan == 0 && D / kSpan >= 1 && D / kSpan <= 6 && D / kSpan != 5;
}

hipError_t launch_fuse_tile(const FuseArgs& a, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream) {
  const int S = a.feat.D / kSpan;
#define AURA_TILE_CASE(s)                                                              \
  case s:                                                                              \
    return a.feat.dtype == 1 ? launch_tile<1, s>(a, tab, n_obj, max_pts, stream)       \
                             : launch_tile<2, s>(a, tab, n_obj, max_pts, stream)
  switch (S) {
    AURA_TILE_CASE(1);
    AURA_TILE_CASE(2);
    AURA_TILE_CASE(3);
    AURA_TILE_CASE(4);
    AURA_TILE_CASE(6);
    default: return hipErrorInvalidValue;
  }
#undef AURA_TILE_CASE
}

}  // namespace aura
