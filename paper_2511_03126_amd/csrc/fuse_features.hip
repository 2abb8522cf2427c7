// aura_fuse_features: Sec. 3.1 "Feature Aggregation", Eq. 2, with the L2 normalisation that the
// cosine similarity of Sec. 3.4.1 implies.
//
// Gather kernel: one wave per point, lanes across the D channels.
//   phase 1  lanes across the views of the point's object: each lane projects the point into one
//            view, evaluates Eq. 1 and prepares the two cell indices and blend weights per axis;
//            a ballot collects the visible views.
//   phase 2  for every visible view (wave-uniform loop over the ballot bits) the four cell rows are
//            read as contiguous D-vectors, widened to fp32 and blended into per-lane accumulators.
//   finish   mean over the visible views, one wave-level sum of squares, scale, streaming store.
// HBM traffic is the compulsory output row (4 D bytes per point) plus each feature cell once;
// the repeated cell reads are served by the caches, which is why points should arrive spatially
// sorted and why workgroup ids are mapped so that each XCD walks a contiguous range of points.
#include "aura_device.hpp"
#include "fuse_args.hpp"
#include "launch.hpp"
#include "timing.hpp"

namespace aura {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int kFuseWaves = 4;
constexpr int kFusePtsPerWave = 8;
constexpr int kFusePtsPerBlock = kFuseWaves * kFusePtsPerWave;

__device__ __forceinline__ void widen_pair(uint32_t w, int dtype_is_bf16, float& lo, float& hi) {
  if (dtype_is_bf16) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xffff0000u);
  } else {
    f16x2 h = __builtin_bit_cast(f16x2, w);
    lo = (float)h[0];
    hi = (float)h[1];
  }
}

// Reads VEC consecutive elements starting at element index e of `base` and widens them to fp32.
// DT: 0 fp32, 1 bf16, 2 fp16.  The address is VEC * sizeof(element) aligned by construction.
template <int DT, int VEC>
__device__ __forceinline__ void load_widen(const void* __restrict__ base, long long e, float (&out)[VEC]) {
  if constexpr (DT == 0) {
    const float* p = static_cast<const float*>(base) + e;
    if constexpr (VEC == 4) {
      f32x4 v = *reinterpret_cast<const f32x4*>(p);
      out[0] = v[0]; out[1] = v[1]; out[2] = v[2]; out[3] = v[3];
    } else if constexpr (VEC == 2) {
      f32x2 v = *reinterpret_cast<const f32x2*>(p);
      out[0] = v[0]; out[1] = v[1];
    } else {
      static_assert(VEC == 1, "fp32 rows are read 1, 2 or 4 elements at a time");
      out[0] = *p;
    }
  } else {
    const uint16_t* p = static_cast<const uint16_t*>(base) + e;
    if constexpr (VEC == 8) {
      u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
      for (int j = 0; j < 4; ++j) widen_pair(v[j], DT == 1, out[2 * j], out[2 * j + 1]);
    } else if constexpr (VEC == 4) {
      u32x2 v = *reinterpret_cast<const u32x2*>(p);
      widen_pair(v[0], DT == 1, out[0], out[1]);
      widen_pair(v[1], DT == 1, out[2], out[3]);
    } else if constexpr (VEC == 2) {
      widen_pair(*reinterpret_cast<const uint32_t*>(p), DT == 1, out[0], out[1]);
    } else {
      static_assert(VEC == 1, "16-bit rows are read 1, 2, 4 or 8 elements at a time");
      float hi;
      widen_pair((uint32_t)*p, DT == 1, out[0], hi);
    }
  }
}

template <int VEC>
__device__ __forceinline__ void store_stream(float* __restrict__ p, const float (&v)[VEC]) {
  if constexpr (VEC % 4 == 0) {
#pragma unroll
    for (int j = 0; j < VEC; j += 4) {
      f32x4 q = {v[j], v[j + 1], v[j + 2], v[j + 3]};
      __builtin_nontemporal_store(q, reinterpret_cast<f32x4*>(p + j));
    }
  } else if constexpr (VEC == 2) {
    f32x2 q = {v[0], v[1]};
    __builtin_nontemporal_store(q, reinterpret_cast<f32x2*>(p));
  } else {
#pragma unroll
    for (int j = 0; j < VEC; ++j) p[j] = v[j];
  }
}

// DT element type, VEC elements per lane per load, PASSES loads per cell row.
// GENERIC == false: D == 64 * VEC * PASSES, the whole row lives in registers.
// GENERIC == true : any D; channels are processed 64 * VEC * PASSES at a time (outer loop), the
//                   unnormalised mean is stored first and rescaled in a second sweep.
template <int DT, int VEC, int PASSES, bool GENERIC>
__global__ __launch_bounds__(kFuseWaves* kWave) void k_fuse_gather(FuseArgs a, ObjTable tab) {
  const ObjRange ob = tab.o[blockIdx.y];
  const int nblk = (ob.n_pts + kFusePtsPerBlock - 1) / kFusePtsPerBlock;
  if ((int)blockIdx.x >= nblk) return;
  const int blk = xcd_contiguous(blockIdx.x, nblk);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  constexpr int CH = kWave * VEC * PASSES;
  const int D = a.feat.D, Hf = a.feat.Hf, Wf = a.feat.Wf;
  const long long view_elems = (long long)Hf * Wf * D;
  const long long elt = DT == 0 ? 4 : 2;

  for (int k = 0; k < kFusePtsPerWave; ++k) {
    const int li = blk * kFusePtsPerBlock + wave * kFusePtsPerWave + k;
    if (li >= ob.n_pts) break;
    const long long i = ob.pt_begin + li;
    const float x = a.xyz[3 * i], y = a.xyz[3 * i + 1], z = a.xyz[3 * i + 2];
    float* __restrict__ out_row = a.fused + i * D;
    float ss = 0.0f;
    int cnt = 0;

    for (int cb = 0; cb < (GENERIC ? D : CH); cb += CH) {
      float acc[PASSES][VEC];
#pragma unroll
      for (int p = 0; p < PASSES; ++p)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[p][e] = 0.0f;
      cnt = 0;

      for (int vb = 0; vb < ob.n_views; vb += kWave) {
        // phase 1: lane j handles view vb + j
        bool seen = false;
        int x0 = 0, y0 = 0;
        float ax = 0.0f, ay = 0.0f;
        if (vb + lane < ob.n_views) {
          const int v = ob.view_begin + vb + lane;
          const Proj p = project(a.vis.cam + (long long)v * 16, x, y, z);
          const float* dv = a.vis.depth ? a.vis.depth + (long long)v * a.vis.H * a.vis.W : nullptr;
          seen = visible(a.vis, dv, p) && view_kept(a, i, vb + lane);
          if (seen) {
            const Tap tx = tap_axis(p.u, a.feat.pitch_x, Wf), ty = tap_axis(p.v, a.feat.pitch_y, Hf);
            x0 = tx.i0; ax = tx.a;
            y0 = ty.i0; ay = ty.a;
          }
        }
        unsigned long long m = __ballot(seen);
        cnt += __popcll(m);
        // phase 2: wave-uniform loop over the visible views
        while (m) {
          const int src = __builtin_ctzll(m);
          m &= m - 1;
          const int sx0 = __builtin_amdgcn_readlane(x0, src), sy0 = __builtin_amdgcn_readlane(y0, src);
          const float sax = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ax), src));
          const float say = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ay), src));
          const int sx1 = sx0 + 1 < Wf ? sx0 + 1 : Wf - 1, sy1 = sy0 + 1 < Hf ? sy0 + 1 : Hf - 1;
          const float w00 = (1.0f - sax) * (1.0f - say), w01 = sax * (1.0f - say);
          const float w10 = (1.0f - sax) * say, w11 = sax * say;
          const char* vbase = static_cast<const char*>(a.feat.feat) +
                              (long long)(ob.view_begin + vb + src) * view_elems * elt;
          const long long o00 = (long long)(sy0 * Wf + sx0) * D, o01 = (long long)(sy0 * Wf + sx1) * D;
          const long long o10 = (long long)(sy1 * Wf + sx0) * D, o11 = (long long)(sy1 * Wf + sx1) * D;
#pragma unroll
          for (int p = 0; p < PASSES; ++p) {
            const int ch = cb + p * kWave * VEC + lane * VEC;
            if (GENERIC && ch >= D) continue;
            float t00[VEC], t01[VEC], t10[VEC], t11[VEC];
            load_widen<DT, VEC>(vbase, o00 + ch, t00);
            load_widen<DT, VEC>(vbase, o01 + ch, t01);
            load_widen<DT, VEC>(vbase, o10 + ch, t10);
            load_widen<DT, VEC>(vbase, o11 + ch, t11);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
              float s = acc[p][e];
              s = __builtin_fmaf(w00, t00[e], s);
              s = __builtin_fmaf(w01, t01[e], s);
              s = __builtin_fmaf(w10, t10[e], s);
              s = __builtin_fmaf(w11, t11[e], s);
              acc[p][e] = s;
            }
          }
        }
      }

      // mean over the visible views (Eq. 2); a point nobody sees keeps zeros
      const float inv = cnt > 0 ? 1.0f / (float)cnt : 0.0f;
#pragma unroll
      for (int p = 0; p < PASSES; ++p)
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          acc[p][e] *= inv;
          ss = __builtin_fmaf(acc[p][e], acc[p][e], ss);
        }
      if constexpr (!GENERIC) {
        float scale = 1.0f;
        if (!a.mean_only) {
          const float nrm = sqrtf(wave_sum(ss));
          scale = 1.0f / fmaxf(nrm, a.norm_eps);
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc[p][e] *= scale;
          store_stream<VEC>(out_row + p * kWave * VEC + lane * VEC, acc[p]);
        }
      } else {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
          const int ch = cb + p * kWave * VEC + lane * VEC;
          if (ch < D) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) out_row[ch + e] = acc[p][e];
          }
        }
      }
    }

    if constexpr (GENERIC) {
      if (!a.mean_only) {
        const float nrm = sqrtf(wave_sum(ss));
        const float scale = 1.0f / fmaxf(nrm, a.norm_eps);
        // every lane rescales exactly the channels it stored above (VEC == 1, PASSES == 1)
        for (int ch = lane; ch < D; ch += kWave) out_row[ch] *= scale;
      }
    }
    if (a.out_count && lane == 0) a.out_count[i] = cnt;
  }
}

template <int DT, int VEC, int PASSES, bool GENERIC>
static hipError_t launch_one(const FuseArgs& a, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream) {
  dim3 grid((max_pts + kFusePtsPerBlock - 1) / kFusePtsPerBlock, n_obj), block(kFuseWaves * kWave);
  const TimingRequest timed = take_timing_request();
  if (timed.start) (void)hipEventRecord(timed.start, stream);
  hipLaunchKernelGGL((k_fuse_gather<DT, VEC, PASSES, GENERIC>), grid, block, 0, stream, a, tab);
  const hipError_t e = hipGetLastError();
  if (timed.stop) (void)hipEventRecord(timed.stop, stream);
  return e;
}

template <int DT>
static hipError_t dispatch_d(const FuseArgs& a, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream) {
  constexpr int V = DT == 0 ? 4 : 8;   // widest load: 16 bytes per lane
  switch (a.feat.D) {
    case 512:  return launch_one<DT, V, 512 / (kWave * V), false>(a, tab, n_obj, max_pts, stream);
    case 768:  return launch_one<DT, 4, 3, false>(a, tab, n_obj, max_pts, stream);
    case 1024: return launch_one<DT, V, 1024 / (kWave * V), false>(a, tab, n_obj, max_pts, stream);
    default:   return launch_one<DT, 1, 1, true>(a, tab, n_obj, max_pts, stream);
  }
}

hipError_t launch_fuse_features(const VisArgs& vis, const FeatArgs& feat, const float* xyz, float* fused,
                                int* out_count, float norm_eps, int mean_only, const TileWs* tile_ws,
                                const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream, float* out_factor,
                                uint8_t* out_vis, int vis_pitch, const uint8_t* in_mask, int in_mask_pitch, int two_kernels,
                                const TileScoring* scoring, bool* scored) {
  if (scored) *scored = false;
  if (n_obj == 0 || max_pts == 0) return hipSuccess;
  FuseArgs a{vis, feat, xyz, fused, out_count, norm_eps, mean_only, tile_ws ? out_factor : nullptr,
             tile_ws ? out_vis : nullptr, vis_pitch, in_mask, in_mask_pitch, two_kernels,
             tile_ws && scoring ? *scoring : TileScoring{}};
  if (tile_ws) return launch_fuse_tile(a, *tile_ws, tab, n_obj, max_pts, stream, scored);
  switch (feat.dtype) {
    case 0: return dispatch_d<0>(a, tab, n_obj, max_pts, stream);
    case 1: return dispatch_d<1>(a, tab, n_obj, max_pts, stream);
    default: return dispatch_d<2>(a, tab, n_obj, max_pts, stream);
  }
}

}  // namespace aura
