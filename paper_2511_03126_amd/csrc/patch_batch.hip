// aura_patch_batch: Sec. 3.2.3 "Multi-scale Feature Fusion", the patches that go to the image encoder.
//
// For every source point, every kept view (aura_select_views) and every scale l, the l x l square of the view's image
// centred at the projection of the point is resampled to R x R (bilinear between pixel centres, border repeated) and
// written channel-first, normalised, into one batch [M][k][L][3][R][R] that the image encoder can take in one call
// (Sec. 3.2, the paragraph on parallelising the semantic feature fusion).
//
// One workgroup per band of 32 rows of a patch.  The workgroup first copies the image pixels the band touches to LDS,
// packed to one word per pixel (a band that touches more than the buffer holds reads the image directly).  A thread
// then takes 4 neighbouring output pixels of a row for all three channels and walks down consecutive rows: column taps
// and weights once; the two horizontally interpolated image rows are reused by all the output rows that fall between
// them, so an output row is one vertical interpolation per value and three 16-byte (fp32) or 8-byte (fp16)
// streaming stores.  The batch is written once and never read here: the call is bound by that
// write (3 R^2 elements per patch).
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

constexpr int kPatchBlock = 256;
constexpr int kPatchMaxScales = 8;
constexpr int kPatchWindow = 4096;      // image pixels of a band of a patch held in LDS (one word each)

struct PatchArgs {
  const float* cam;
  const uint8_t* images;   // [n_views][H][W][3]
  int H, W;
  const float* xyz;
  const int* sel_view;     // [M][k]
  int k, L, R;
  int band;                // output rows per workgroup
  float scales[kPatchMaxScales];
  float scale[3], offset[3];   // stored value = pixel value * scale[c] + offset[c]: inv_std / 255 and -mean * inv_std
  void* out;               // [M][k][L][3][R][R]
  uint8_t* valid;          // [M][k] or nullptr
};

typedef float patch_f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 patch_f16x4 __attribute__((ext_vector_type(4)));

// HALF: fp16 output.  VEC: output pixels per thread and trip (4 when R % 4 == 0, else 1).
// A workgroup produces a band of `band` rows of one patch (bands keep the number of workgroups well above what the
// chip holds at once, so its last round is nearly full).  Thread t owns output columns VEC (t % per_row) .. + VEC - 1 and
// walks down the band's rows: everything that depends on the column only (taps, weights) is computed once.
template <bool HALF, int VEC>
__global__ __launch_bounds__(kPatchBlock) void k_patch_batch(PatchArgs a, ObjTable tab) {
  __shared__ uint32_t s_win[kPatchWindow];
  const ObjRange ob = tab.o[blockIdx.y];
  const int R = a.R;
  const int n_bands = (R + a.band - 1) / a.band;
  const int per_point = a.k * a.L * n_bands;
  if ((long long)blockIdx.x >= (long long)ob.n_pts * per_point) return;
  const int lp = blockIdx.x / per_point, rest = blockIdx.x % per_point;
  const int rl = rest / n_bands, band = rest % n_bands;
  const int rank = rl / a.L, l = rl % a.L;
  const long long s = ob.pt_begin + lp;
  const int sv = a.sel_view[s * a.k + rank];
  const bool ok = sv >= 0 && sv < ob.n_views;
  if (a.valid && l == 0 && band == 0 && threadIdx.x == 0) a.valid[s * a.k + rank] = ok ? 1 : 0;
  const long long plane = (long long)R * R;
  const long long patch0 = ((s * a.k + rank) * a.L + l) * 3 * plane;   // first element of the patch
  const int i_lo = band * a.band, i_hi = min(R, i_lo + a.band);          // rows of this workgroup

  float u = 0.0f, v = 0.0f;
  const uint8_t* __restrict__ img = a.images;
  if (ok) {
    const int view = ob.view_begin + sv;
    const Proj p = project(a.cam + (long long)view * 16, a.xyz[3 * s], a.xyz[3 * s + 1], a.xyz[3 * s + 2]);
    u = p.u;
    v = p.v;
    img += (long long)view * a.H * a.W * 3;
  }
  const float side = a.scales[l];
  const float step = side / (float)R;
  const float x_first = u - 0.5f * side, y_first = v - 0.5f * side;
  const float wmax = (float)(a.W - 1), hmax = (float)(a.H - 1);
  // texel coordinate of output column j / row i: pixel centres at integer + 0.5, clamped to the image (border repeated)
  auto texel_x = [&](int j) { return fminf(fmaxf(__builtin_fmaf((float)j + 0.5f, step, x_first) - 0.5f, 0.0f), wmax); };
  auto texel_y = [&](int i) { return fminf(fmaxf(__builtin_fmaf((float)i + 0.5f, step, y_first) - 0.5f, 0.0f), hmax); };

  // The part of the image that the band touches: columns wx0 .. wx0 + ww - 1, rows wy0 .. wy0 + wh - 1 (the sample
  // positions grow with j and i, so the first and the last output pixel bound it).  When it fits, the workgroup copies
  // it to LDS once, one 32-bit word per pixel (three channels), and a tap is one LDS read instead of three byte reads
  // from memory.
  int wx0 = 0, wy0 = 0, ww = 0;
  bool staged = false;
  if (ok) {
    wx0 = (int)floorf(texel_x(0));
    wy0 = (int)floorf(texel_y(i_lo));
    ww = min((int)floorf(texel_x(R - 1)) + 1, a.W - 1) - wx0 + 1;
    const int wh = min((int)floorf(texel_y(i_hi - 1)) + 1, a.H - 1) - wy0 + 1;
    staged = (long long)ww * wh <= kPatchWindow;      // uniform over the workgroup
    if (staged) {
      for (int t = threadIdx.x; t < ww * wh; t += kPatchBlock) {
        const int wy = t / ww, wx = t % ww;
        const uint8_t* __restrict__ px = img + ((long long)(wy0 + wy) * a.W + (wx0 + wx)) * 3;
        s_win[t] = (uint32_t)px[0] | ((uint32_t)px[1] << 8) | ((uint32_t)px[2] << 16);
      }
    }
  }
  __syncthreads();

  const int per_row = R / VEC;
  // thread -> (row within a trip, column group); with more column groups than threads a thread takes several
  const int rows_per_trip = per_row <= kPatchBlock ? kPatchBlock / per_row : 1;
  const int my_row = per_row <= kPatchBlock ? threadIdx.x / per_row : 0;
  if (my_row >= rows_per_trip) return;              // threads beyond the last full row of a trip (after the barrier)
  for (int cg = per_row <= kPatchBlock ? threadIdx.x % per_row : threadIdx.x; cg < per_row; cg += kPatchBlock) {
    const int j0 = cg * VEC;
    int x0[VEC], x1[VEC];
    float ax[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const float gx = texel_x(j0 + e);
      const float fx = floorf(gx);
      x0[e] = (int)fx;
      x1[e] = x0[e] + 1 < a.W ? x0[e] + 1 : a.W - 1;
      ax[e] = gx - fx;
    }
    // The thread's rows are consecutive.  Several output rows fall between the same two image rows (the patch is
    // magnified), so the two horizontally interpolated image rows are kept and only replaced when the output row
    // moves on to the next image row; an output row then costs one vertical interpolation per value.
    const int chunk = (i_hi - i_lo + rows_per_trip - 1) / rows_per_trip;
    const int r_lo = i_lo + my_row * chunk, r_hi = min(i_hi, r_lo + chunk);
    float top[3][VEC], bot[3][VEC];
    int top_y = -1, bot_y = -1;          // image rows held in top / bot
    auto image_row = [&](int y, float (&dst)[3][VEC]) {
      const uint8_t* __restrict__ row = img + (long long)y * a.W * 3;
      const int rr = (y - wy0) * ww - wx0;                      // LDS index of image column 0 of the row
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        uint32_t pa, pb;
        if (staged) {
          pa = s_win[rr + x0[e]];
          pb = s_win[rr + x1[e]];
        } else {
          pa = (uint32_t)row[3 * x0[e]] | ((uint32_t)row[3 * x0[e] + 1] << 8) | ((uint32_t)row[3 * x0[e] + 2] << 16);
          pb = (uint32_t)row[3 * x1[e]] | ((uint32_t)row[3 * x1[e] + 1] << 8) | ((uint32_t)row[3 * x1[e] + 2] << 16);
        }
#pragma unroll
        for (int c = 0; c < 3; ++c) {
          const float ta = (float)((pa >> (8 * c)) & 0xffu), tb = (float)((pb >> (8 * c)) & 0xffu);
          dst[c][e] = __builtin_fmaf(ax[e], tb - ta, ta);
        }
      }
    };
    for (int i = r_lo; i < r_hi; ++i) {
      float val[3][VEC];
      if (ok) {
        const float gy = texel_y(i);
        const float fy = floorf(gy);
        const int y0 = (int)fy, y1 = y0 + 1 < a.H ? y0 + 1 : a.H - 1;
        const float ay = gy - fy;
        if (y0 != top_y) {
          if (y0 == bot_y) {
#pragma unroll
            for (int c = 0; c < 3; ++c)
#pragma unroll
              for (int e = 0; e < VEC; ++e) top[c][e] = bot[c][e];
          } else {
            image_row(y0, top);
          }
          top_y = y0;
        }
        if (y1 != bot_y) {
          image_row(y1, bot);
          bot_y = y1;
        }
#pragma unroll
        for (int c = 0; c < 3; ++c)
#pragma unroll
          for (int e = 0; e < VEC; ++e)
            val[c][e] = __builtin_fmaf(__builtin_fmaf(ay, bot[c][e] - top[c][e], top[c][e]), a.scale[c], a.offset[c]);
      } else {
#pragma unroll
        for (int c = 0; c < 3; ++c)
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[c][e] = 0.0f;
      }
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        const long long o = patch0 + c * plane + (long long)i * R + j0;
        if constexpr (VEC == 4) {
          if constexpr (HALF) {
            const patch_f16x4 h = {(_Float16)val[c][0], (_Float16)val[c][1], (_Float16)val[c][2], (_Float16)val[c][3]};
            __builtin_nontemporal_store(h, reinterpret_cast<patch_f16x4*>(static_cast<_Float16*>(a.out) + o));
          } else {
            const patch_f32x4 f = {val[c][0], val[c][1], val[c][2], val[c][3]};
            __builtin_nontemporal_store(f, reinterpret_cast<patch_f32x4*>(static_cast<float*>(a.out) + o));
          }
        } else {
          if constexpr (HALF) static_cast<_Float16*>(a.out)[o] = (_Float16)val[c][0];
          else static_cast<float*>(a.out)[o] = val[c][0];
        }
      }
    }
  }
}

bool patch_batch_supported(int L) { return L >= 1 && L <= kPatchMaxScales; }

hipError_t launch_patch_batch(const float* cam, const uint8_t* images, int H, int W, const float* xyz, const int* sel_view,
                              int k, const float* scales, int L, int R, const float* mean, const float* inv_std,
                              void* out, bool half, uint8_t* valid, const ObjTable& tab, int n_obj, int max_pts,
                              hipStream_t stream) {
  if (n_obj == 0 || max_pts == 0) return hipSuccess;
  PatchArgs a{};
  a.cam = cam; a.images = images; a.H = H; a.W = W; a.xyz = xyz; a.sel_view = sel_view; a.k = k; a.L = L; a.R = R;
  for (int l = 0; l < L; ++l) a.scales[l] = scales[l];
  for (int c = 0; c < 3; ++c) {
    const float mu = mean ? mean[c] : 0.0f, is = inv_std ? inv_std[c] : 1.0f;
    a.scale[c] = is / 255.0f;
    a.offset[c] = -mu * is;
  }
  a.out = out; a.valid = valid;
  a.band = R < 32 ? R : 32;
  const int n_bands = (R + a.band - 1) / a.band;
  const dim3 grid((unsigned)((long long)max_pts * k * L * n_bands), n_obj), block(kPatchBlock);
  // 16-byte (fp32) / 8-byte (fp16) stores need R % 4 == 0 and a base aligned alike
  const bool vec = R % 4 == 0 && (reinterpret_cast<uintptr_t>(out) & (half ? 7 : 15)) == 0;
  if (half) {
    if (vec) hipLaunchKernelGGL((k_patch_batch<true, 4>), grid, block, 0, stream, a, tab);
    else hipLaunchKernelGGL((k_patch_batch<true, 1>), grid, block, 0, stream, a, tab);
  } else {
    if (vec) hipLaunchKernelGGL((k_patch_batch<false, 4>), grid, block, 0, stream, a, tab);
    else hipLaunchKernelGGL((k_patch_batch<false, 1>), grid, block, 0, stream, a, tab);
  }
  return hipGetLastError();
}

}  // namespace aura
