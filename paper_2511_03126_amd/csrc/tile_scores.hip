// aura_fuse_scores, scoring part (Sec. 3.4.1) on top of the matrix-core fusion path.
//
// The similarity omega_k = <f, t_k> is linear in the feature, and the fused feature of Eq. 2 is a
// weighted sum of feature cells, f_i = s_i * sum_c w[i][c] F[c] (s_i: 1 / (count * norm)).  Hence
//     omega[i][k] = s_i * sum_c w[i][c] * G[c][k],      G[c][k] = <F[c], t_k>,
// i.e. the same tile product as the fusion itself, but over K "channels" instead of D.  Where a call
// has fewer feature cells than points, G is cheap (one small dense product per call) and the scores
// never need the fused rows to be read back from memory:
//
//   k_cell_scores   G = F . T^T for every cell of every view, on the matrix cores, fp32 accumulate, the
//                   text embeddings split into two 16-bit terms; stored as two 16-bit terms per value.
//   k_tile_scores   one wave per 32-point tile: omega^T = G^T . W^T over the tile's k-steps as written
//                   by the prepare kernel (its weight operand is exactly the B operand here), three
//                   partial products per k-step (hi*hi, hi*lo, lo*hi), times the point's factor s_i that the
//                   product kernel left in the workspace; then the shared epilogue (scores, label, Eq. 4).
//
// A tile that the fusion kernel fused by a per-point gather (no k-steps) was scored there as well.
#include "aura_device.hpp"
#include "fuse_args.hpp"
#include "launch.hpp"
#include "scores_epilogue.hpp"
#include "tile_scores.hpp"

namespace aura {

typedef __bf16 ts_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 ts_f16x8 __attribute__((ext_vector_type(8)));
typedef float ts_f32x4 __attribute__((ext_vector_type(4)));
typedef float ts_f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t ts_u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ ts_f32x16 ts_mma(ts_u32x4 a, ts_u32x4 b, ts_f32x16 c) {
  if constexpr (DT == 1)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(ts_bf16x8, a), __builtin_bit_cast(ts_bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(ts_f16x8, a), __builtin_bit_cast(ts_f16x8, b), c, 0, 0, 0);
}

// x = hi + lo with both terms in the 16-bit type of the feature maps; returns hi | lo << 16.
template <int DT>
__device__ __forceinline__ uint32_t split_pack(float x) {
  if constexpr (DT == 1) {
    const __bf16 h = (__bf16)x;
    const __bf16 l = (__bf16)(x - (float)h);
    return (uint32_t)__builtin_bit_cast(uint16_t, h) | ((uint32_t)__builtin_bit_cast(uint16_t, l) << 16);
  } else {
    const _Float16 h = (_Float16)x;
    const _Float16 l = (_Float16)(x - (float)h);
    return (uint32_t)__builtin_bit_cast(uint16_t, h) | ((uint32_t)__builtin_bit_cast(uint16_t, l) << 16);
  }
}

// ------------------------------------------------------------------------------------ G = F . T^T

struct CellArgs {
  const char* feat;     // [n_cells][D] 16-bit
  long long n_cells;
  int D, K, Kpad;
  const float* temb;    // [K][D] fp32
  uint32_t* G;          // [n_cells][Kpad]: hi | lo << 16
  ts_u32x4* t_split;    // the text embeddings as matrix-core operands: [D / 16][Kpad / 32][hi, lo][64 lanes] x 16 bytes
};

// The text embeddings split into two terms of the maps' 16-bit type, once per call, in the order in which the lanes of
// k_cell_scores take them: lane (material n = l % 32, kg = l / 32) of slot (step s, tile mt) holds channels
// 16 s + 8 kg .. + 7 of material 32 mt + n (zeros beyond K).
template <int DT>
__global__ __launch_bounds__(256) void k_split_for_cells(CellArgs a) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;   // one thread per (step, tile, lane)
  const int MT = a.Kpad / 32;
  if (t >= (long long)(a.D / 16) * MT * kWave) return;
  const int lane = (int)(t % kWave), mt = (int)((t / kWave) % MT), s = (int)(t / ((long long)kWave * MT));
  const int n = mt * 32 + (lane & 31), kg = lane >> 5;
  uint32_t p[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) p[e] = split_pack<DT>(n < a.K ? a.temb[(long long)n * a.D + s * 16 + kg * 8 + e] : 0.0f);
  ts_u32x4 hi, lo;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    hi[q] = __builtin_amdgcn_perm(p[2 * q + 1], p[2 * q], 0x05040100u);
    lo[q] = __builtin_amdgcn_perm(p[2 * q + 1], p[2 * q], 0x07060302u);
  }
  ts_u32x4* slot = a.t_split + ((long long)(s * MT + mt) * 2) * kWave + lane;
  slot[0] = hi;
  slot[kWave] = lo;
}

// One workgroup of four waves per 128 cells, all materials, all channels: wave w multiplies the rows of cells
// 32 w .. 32 w + 31.  The table above passes through LDS in chunks of 16 KiB (8 / MT groups of 16 channels), double
// buffered (four workgroups fit a compute unit): the workgroup copies the next chunk in while it multiplies with this one, so the table comes from L2 once per
// 128 cells (with one workgroup per 32 cells, every wave reading its operands from L2, it was 16 KiB of table per cell
// against 2 KiB of features for 1024 channels and 128 materials, and a 48 KiB buffer for the partial sums held a compute
// unit to three workgroups).  A operand: lane (cell i = l % 32, kg = l / 32) holds channels 16 s + 8 kg .. + 7 of cell i
// (16 contiguous bytes of the stored map), requested one chunk ahead; B operand: the same channels of material
// n = l % 32.  One chain of partial sums per (cell, material): channel groups in ascending order, hi then lo.
template <int DT, int MT>
__global__ __launch_bounds__(256) void k_cell_scores(CellArgs a) {
  constexpr int CS = 8 / MT;                    // groups of 16 channels per chunk
  constexpr int kChunkVecs = 8 * 2 * kWave;     // 16-byte units per chunk: CS * MT slots of hi and lo
  constexpr int kCopies = kChunkVecs / 256;     // per thread
  __shared__ ts_u32x4 s_tab[2][kChunkVecs];
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const long long c0 = (long long)blockIdx.x * 128 + wave * 32;
  const int i = lane & 31, kg = lane >> 5;
  const long long cell = min(c0 + i, a.n_cells - 1);
  const char* __restrict__ frow = a.feat + cell * a.D * 2 + kg * 16;
  const int n_chunks = a.D / (16 * CS);

  ts_f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;

  ts_u32x4 tab_r[kCopies], f_cur[CS], f_nxt[CS];
#pragma unroll
  for (int v = 0; v < kCopies; ++v) tab_r[v] = a.t_split[v * 256 + tid];
#pragma unroll
  for (int q = 0; q < CS; ++q) f_cur[q] = *reinterpret_cast<const ts_u32x4*>(frow + q * 32);
#pragma unroll
  for (int v = 0; v < kCopies; ++v) s_tab[0][v * 256 + tid] = tab_r[v];
  __syncthreads();

  for (int c = 0; c < n_chunks; ++c) {
    const bool more = c + 1 < n_chunks;
    if (more) {
#pragma unroll
      for (int v = 0; v < kCopies; ++v) tab_r[v] = a.t_split[(long long)(c + 1) * kChunkVecs + v * 256 + tid];
#pragma unroll
      for (int q = 0; q < CS; ++q) f_nxt[q] = *reinterpret_cast<const ts_u32x4*>(frow + ((c + 1) * CS + q) * 32);
    }
    const ts_u32x4* tab = s_tab[c & 1];
#pragma unroll
    for (int q = 0; q < CS; ++q) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const ts_u32x4 bh = tab[((q * MT + mt) * 2) * kWave + lane], bl = tab[((q * MT + mt) * 2 + 1) * kWave + lane];
        acc[mt] = ts_mma<DT>(f_cur[q], bh, acc[mt]);
        acc[mt] = ts_mma<DT>(f_cur[q], bl, acc[mt]);
      }
    }
    if (more) {   // nobody reads the other buffer between the previous trip's barrier and this trip's
#pragma unroll
      for (int v = 0; v < kCopies; ++v) s_tab[(c + 1) & 1][v * 256 + tid] = tab_r[v];
#pragma unroll
      for (int q = 0; q < CS; ++q) f_cur[q] = f_nxt[q];
    }
    __syncthreads();
  }
  // element r of the lane: cell c0 + 8 (r / 4) + 4 kg + r % 4, material 32 mt + i (0 beyond K)
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const long long c = c0 + 8 * (r >> 2) + 4 * kg + (r & 3);
      const float v = (mt * 32 + i < a.K) ? acc[mt][r] : 0.0f;
      if (c < a.n_cells) a.G[c * a.Kpad + mt * 32 + i] = split_pack<DT>(v);
    }
}

// The same with the embeddings split by every wave on the fly (B operand: the channels of material n = l % 32 read as
// fp32 and split in registers): no table and no launch to build it, which is what counts for calls with few cells
// (16 384 cells: 12 us for this kernel alone, while the launch that builds the table costs 5 us by itself).
template <int DT, int MT>
__global__ __launch_bounds__(256) void k_cell_scores_small(CellArgs a) {
  __shared__ float s_part[3][MT][16][kWave];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const long long c0 = (long long)blockIdx.x * 32;
  const int i = lane & 31, kg = lane >> 5;
  const long long cell = min(c0 + i, a.n_cells - 1);
  const char* __restrict__ frow = a.feat + cell * a.D * 2 + kg * 16;
  const float* __restrict__ trow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) trow[mt] = a.temb + (long long)min(mt * 32 + i, a.K - 1) * a.D + kg * 8;

  ts_f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;

  for (int s = wave; s < a.D / 16; s += 4) {
    const ts_u32x4 fa = *reinterpret_cast<const ts_u32x4*>(frow + s * 32);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const ts_f32x4 t0 = *reinterpret_cast<const ts_f32x4*>(trow[mt] + s * 16);
      const ts_f32x4 t1 = *reinterpret_cast<const ts_f32x4*>(trow[mt] + s * 16 + 4);
      const float t[8] = {t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3]};
      ts_u32x4 bh, bl;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t p0 = split_pack<DT>(t[2 * q]), p1 = split_pack<DT>(t[2 * q + 1]);
        bh[q] = __builtin_amdgcn_perm(p1, p0, 0x05040100u);
        bl[q] = __builtin_amdgcn_perm(p1, p0, 0x07060302u);
      }
      acc[mt] = ts_mma<DT>(fa, bh, acc[mt]);
      acc[mt] = ts_mma<DT>(fa, bl, acc[mt]);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_part[wave - 1][mt][r][lane] = acc[mt][r];
  }
  __syncthreads();
  if (wave > 0) return;
  // element r of the lane: cell c0 + 8 (r / 4) + 4 kg + r % 4, material 32 mt + i (0 beyond K)
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const long long c = c0 + 8 * (r >> 2) + 4 * kg + (r & 3);
      const float sum = ((acc[mt][r] + s_part[0][mt][r][lane]) + s_part[1][mt][r][lane]) + s_part[2][mt][r][lane];
      const float v = (mt * 32 + i < a.K) ? sum : 0.0f;
      if (c < a.n_cells) a.G[c * a.Kpad + mt * 32 + i] = split_pack<DT>(v);
    }
}

// ------------------------------------------------------------------------------------ per-tile scores

struct TileScoreArgs {
  const TileHdr* hdr;
  const TileStep* steps;
  int quota;
  const uint32_t* G;
  int Kpad;
  uint32_t row_units;    // D / 256
  const float* factor;   // [N]
  int D, K, P;
  const float* y;
  float inv_T;
  int unseen_zero;
  float* scores;
  float* prop;
  int* label;
};

template <int DT, int MT>
__global__ __launch_bounds__(256) void k_tile_scores(TileScoreArgs a, ObjTable tab) {
  __shared__ float ys[kScoreMaxK * kScoreMaxP];
  __shared__ __attribute__((aligned(16))) float s_stage[4][score_stage_floats<16>()];
  const ObjRange ob = tab.o[blockIdx.y];
  const int nblk = (ob.n_pts + kTilePts - 1) / kTilePts;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int tile = blockIdx.x * 4 + wave;
  const int nsteps = tile < nblk ? a.hdr[ob.tile_begin + tile].nsteps : -1;
  // Nothing to do here for a tile fused by a gather inside the fusion kernel (nsteps < 0: scored there as well) and for
  // a tile that no view sees (k_tile_zero_rows writes its results); a workgroup of such tiles leaves at once.
  const bool mine = nsteps > 0 || (nsteps == 0 && !(0.0f * a.inv_T == 0.0f));
  if (!__syncthreads_or(mine)) return;
  if (a.prop) {
    for (int t = threadIdx.x; t < a.K * a.P; t += blockDim.x) ys[t] = a.y[t];
  }
  __syncthreads();
  if (!mine) return;
  const int pt = lane & 31, g = lane >> 5;
  const int li = tile * kTilePts + pt;
  const bool valid = li < ob.n_pts;
  const long long n = ob.pt_begin + (valid ? li : ob.n_pts - 1);

  ts_f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;

  const TileStep* __restrict__ st = a.steps + (long long)(ob.tile_begin + tile) * a.quota;
  for (int s = 0; s < nsteps; ++s) {
    const ts_u32x4 w_hi = st[s].a_hi[lane], w_lo = st[s].a_lo[lane];
    const ts_u32x4 c0 = *reinterpret_cast<const ts_u32x4*>(&st[s].cell[8 * g]);
    const ts_u32x4 c1 = *reinterpret_cast<const ts_u32x4*>(&st[s].cell[8 * g + 4]);
    uint32_t gv[MT][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t ci = cell_index(e < 4 ? c0[e] : c1[e - 4], a.row_units);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) gv[mt][e] = a.G[(long long)ci * a.Kpad + mt * 32 + pt];
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      ts_u32x4 g_hi, g_lo;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        g_hi[q] = __builtin_amdgcn_perm(gv[mt][2 * q + 1], gv[mt][2 * q], 0x05040100u);
        g_lo[q] = __builtin_amdgcn_perm(gv[mt][2 * q + 1], gv[mt][2 * q], 0x07060302u);
      }
      acc[mt] = ts_mma<DT>(g_hi, w_hi, acc[mt]);
      acc[mt] = ts_mma<DT>(g_hi, w_lo, acc[mt]);
      acc[mt] = ts_mma<DT>(g_lo, w_hi, acc[mt]);
    }
  }
  const float f = a.factor[n];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] *= f;
  finish_scores_staged<MT, 16>(acc, ob.pt_begin + (long long)tile * kTilePts, min(kTilePts, ob.n_pts - tile * kTilePts), lane,
                               a.K, a.P, a.inv_T, ys, a.scores, a.prop, a.label, a.unseen_zero != 0, s_stage[wave]);
}

// The tiles that no view sees (the inside of a solid: 9 of 10 tiles of a voxelised body): every similarity is +0 and the
// result is known without the products and the exponentials - scores 0, label 0, the properties of Eq. 4 on equal
// similarities.  A kernel of its own because it is nothing but stores and wants many waves in flight, while the scoring
// kernel with 128 materials holds three waves per SIMD.  One wave per tile; workgroups without such a tile leave at once.
template <int MT>
__global__ __launch_bounds__(256) void k_tile_zero_rows(TileScoreArgs a, ObjTable tab) {
  __shared__ float ys[kScoreMaxK * kScoreMaxP];
  const ObjRange ob = tab.o[blockIdx.y];
  const int nblk = (ob.n_pts + kTilePts - 1) / kTilePts;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int tile = blockIdx.x * 4 + wave;
  const bool mine = tile < nblk && a.hdr[ob.tile_begin + (tile < nblk ? tile : 0)].nsteps == 0 && 0.0f * a.inv_T == 0.0f;
  if (!__syncthreads_or(mine)) return;
  if (a.prop) {
    for (int t = threadIdx.x; t < a.K * a.P; t += blockDim.x) ys[t] = a.y[t];
  }
  __syncthreads();
  if (!mine) return;
  finish_zero_rows<MT>(ob.pt_begin + (long long)tile * kTilePts, min(kTilePts, ob.n_pts - tile * kTilePts), lane, a.K, a.P, ys,
                       a.scores, a.prop, a.label, a.unseen_zero != 0);
}

// ------------------------------------------------------------------------------------ host

static size_t ts_round256(size_t x) { return (x + 255) & ~(size_t)255; }
static int ts_kpad(int K) {
  int mt = (K + 31) / 32;
  if (mt == 3) mt = 4;
  return mt * 32;
}

// the split text embeddings for the largest channel count of the matrix-core path (1536)
static size_t ts_split_bytes(int K) { return (size_t)(1536 / 16) * (ts_kpad(K) / 32) * 2 * kWave * 16; }

size_t tile_scores_workspace_bytes(long long N, long long n_cells, int K) {
  return ts_round256((size_t)N * sizeof(float)) + ts_round256((size_t)n_cells * ts_kpad(K) * sizeof(uint32_t)) +
         ts_split_bytes(K);
}

TileScoreWs tile_scores_workspace(void* workspace, long long N, long long n_cells, int K) {
  TileScoreWs ws;
  char* base = static_cast<char*>(workspace);
  ws.factor = reinterpret_cast<float*>(base);
  base += ts_round256((size_t)N * sizeof(float));
  ws.G = reinterpret_cast<uint32_t*>(base);
  base += ts_round256((size_t)n_cells * ts_kpad(K) * sizeof(uint32_t));
  ws.t_split = base;
  ws.Kpad = ts_kpad(K);
  return ws;
}

template <int DT>
static hipError_t launch_cells(const CellArgs& a, hipStream_t stream) {
  if (a.n_cells * (a.Kpad / 32) < 32768) {
    const dim3 grid((unsigned)((a.n_cells + 31) / 32)), block(256);
    switch (a.Kpad / 32) {
      case 1: hipLaunchKernelGGL((k_cell_scores_small<DT, 1>), grid, block, 0, stream, a); break;
      case 2: hipLaunchKernelGGL((k_cell_scores_small<DT, 2>), grid, block, 0, stream, a); break;
      default: hipLaunchKernelGGL((k_cell_scores_small<DT, 4>), grid, block, 0, stream, a); break;
    }
    return hipGetLastError();
  }
  const long long slots = (long long)(a.D / 16) * (a.Kpad / 32) * kWave;
  hipLaunchKernelGGL((k_split_for_cells<DT>), dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, stream, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)((a.n_cells + 127) / 128)), block(256);
  switch (a.Kpad / 32) {
    case 1: hipLaunchKernelGGL((k_cell_scores<DT, 1>), grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL((k_cell_scores<DT, 2>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((k_cell_scores<DT, 4>), grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

hipError_t launch_cell_scores(const FeatArgs& feat, long long n_cells, const float* temb, int K, const TileScoreWs& ws,
                              hipStream_t stream) {
  CellArgs a{static_cast<const char*>(feat.feat), n_cells, feat.D, K, ws.Kpad, temb, ws.G, static_cast<ts_u32x4*>(ws.t_split)};
  return feat.dtype == 1 ? launch_cells<1>(a, stream) : launch_cells<2>(a, stream);
}

template <int DT>
static hipError_t launch_ts(const TileScoreArgs& a, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream) {
  const int max_tiles = (max_pts + kTilePts - 1) / kTilePts;
  const dim3 grid((unsigned)((max_tiles + 3) / 4), (unsigned)n_obj), block(256);
  switch (a.Kpad / 32) {
    case 1: hipLaunchKernelGGL((k_tile_zero_rows<1>), grid, block, 0, stream, a, tab); break;
    case 2: hipLaunchKernelGGL((k_tile_zero_rows<2>), grid, block, 0, stream, a, tab); break;
    default: hipLaunchKernelGGL((k_tile_zero_rows<4>), grid, block, 0, stream, a, tab); break;
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  switch (a.Kpad / 32) {
    case 1: hipLaunchKernelGGL((k_tile_scores<DT, 1>), grid, block, 0, stream, a, tab); break;
    case 2: hipLaunchKernelGGL((k_tile_scores<DT, 2>), grid, block, 0, stream, a, tab); break;
    default: hipLaunchKernelGGL((k_tile_scores<DT, 4>), grid, block, 0, stream, a, tab); break;
  }
  return hipGetLastError();
}

hipError_t launch_tile_scores(const FeatArgs& feat, const TileWs& tws, const TileScoreWs& ws,
                              int K, const float* y, int P, float temperature, int unseen_zero, float* scores,
                              float* prop, int* label, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream) {
  TileScoreArgs a{tws.hdr, tws.steps, tws.quota, ws.G, ws.Kpad, (uint32_t)(feat.D / 256), ws.factor,
                  feat.D, K, P, y, 1.0f / temperature, unseen_zero, scores, prop, label};
  return feat.dtype == 1 ? launch_ts<1>(a, tab, n_obj, max_pts, stream) : launch_ts<2>(a, tab, n_obj, max_pts, stream);
}

}  // namespace aura
