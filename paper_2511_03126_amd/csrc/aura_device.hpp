// Shared device-side pieces of libaura_fuse (gfx950, wave64).
//
// The projection / visibility / cell-selection functions below are the single definition of
// the fp32 decision arithmetic (Sec. 3.1, Eq. 1 of the AURA paper): every kernel that needs the
// mask or the sampled cells calls these, so all entry points agree bit for bit.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aura {

constexpr int kWave = 64;
constexpr int kMaxObjPerLaunch = 64;   // objects described by one kernel-argument table

// One object of a launch: its point range and its view range.
struct ObjRange {
  long long pt_begin;
  int n_pts;
  int view_begin;
  int n_views;
  int tile_begin;   // index of the object's first 32-point tile within the call
};

struct ObjTable {
  ObjRange o[kMaxObjPerLaunch];
};

// What Eq. 1 needs besides the point.
struct VisArgs {
  const float* cam;     // [n_views][16]
  const float* depth;   // [n_views][H][W] or nullptr (frustum only)
  int H, W;
  float tau, z_near;
  int frustum_only;
};

// Workgroups are handed to the 8 XCDs round-robin by linear id.  This maps the id so that each
// XCD walks one contiguous range of work items, which keeps neighbouring (spatially sorted)
// points, and the feature cells they share, in one XCD's L2.
__device__ __forceinline__ int xcd_contiguous(int bid, int nblk) {
  constexpr int kXcd = 8;
  int xcd = bid % kXcd, idx = bid / kXcd;
  int per = nblk / kXcd, rem = nblk % kXcd;
  return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

struct Proj {
  float u, v, z;
};

// pi(x, v) and proj_depth: Xc = R x + t as a chain of fused multiply-adds starting from t, one
// IEEE division per pixel coordinate, one fused multiply-add with the focal length.
// CamPtr: a pointer to the 16 floats of a camera row in any address space (memory or LDS).
template <typename CamPtr>
__device__ __forceinline__ Proj project(CamPtr c, float x, float y, float z) {
#pragma clang fp contract(off)
  float xc = __builtin_fmaf(c[2], z, __builtin_fmaf(c[1], y, __builtin_fmaf(c[0], x, c[9])));
  float yc = __builtin_fmaf(c[5], z, __builtin_fmaf(c[4], y, __builtin_fmaf(c[3], x, c[10])));
  float zc = __builtin_fmaf(c[8], z, __builtin_fmaf(c[7], y, __builtin_fmaf(c[6], x, c[11])));
  float qx = xc / zc;
  float qy = yc / zc;
  Proj p;
  p.u = __builtin_fmaf(c[12], qx, c[14]);
  p.v = __builtin_fmaf(c[13], qy, c[15]);
  p.z = zc;
  return p;
}

// M_vis of Eq. 1 (with the tolerance tau), in three steps so that a kernel may issue the depth
// read early: (1) in front of the camera and inside the image, (2) which texel, (3) the comparison.
__device__ __forceinline__ bool in_frustum(const VisArgs& a, const Proj& p) {
  return (p.z > a.z_near) && (p.u >= 0.0f) && (p.u < (float)a.W) && (p.v >= 0.0f) && (p.v < (float)a.H);
}

// Only meaningful when in_frustum() holds.
__device__ __forceinline__ int depth_texel(const VisArgs& a, const Proj& p) {
  int px = (int)floorf(p.u), py = (int)floorf(p.v);
  return py * a.W + px;
}

__device__ __forceinline__ bool passes_depth(const VisArgs& a, const Proj& p, float d) {
#pragma clang fp contract(off)
  if (!(d > 0.0f)) return false;
  float lim = d + a.tau;
  return p.z <= lim;
}

__device__ __forceinline__ bool visible(const VisArgs& a, const float* __restrict__ depth_v, const Proj& p) {
  if (!in_frustum(a, p)) return false;
  if (a.frustum_only) return true;
  return passes_depth(a, p, depth_v[depth_texel(a, p)]);
}

// The two cells around grid coordinate g = coord / pitch - 0.5 (clamped) and the weight of the
// second one.
struct Tap {
  int i0, i1;
  float a;
};

__device__ __forceinline__ Tap tap_axis(float coord, float pitch, int size_grid) {
#pragma clang fp contract(off)
  float q = coord / pitch;
  float g = q - 0.5f;
  g = fminf(fmaxf(g, 0.0f), (float)(size_grid - 1));
  float fl = floorf(g);
  Tap t;
  t.i0 = (int)fl;
  t.i1 = (t.i0 + 1 < size_grid) ? t.i0 + 1 : size_grid - 1;
  t.a = g - fl;
  return t;
}

// exp(x) for the weights of Eq. 4 (x <= 0: a similarity minus the row's largest, over T): the hardware's base-2
// exponential of x * log2(e).  Two instructions where the library routine takes about thirty; the product's rounding
// costs a weight of exp(-20) a relative 2e-6 and the large weights nothing, far inside what Eq. 4 in fp32 holds anyway
// (the epilogues of the scoring kernels spend most of their instructions here: 64 exponentials per lane with 128
// materials).  exp(+0) is exactly 1.
__device__ __forceinline__ float weight_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896340736f); }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

__device__ __forceinline__ long long wave_sum(long long x) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

}  // namespace aura
