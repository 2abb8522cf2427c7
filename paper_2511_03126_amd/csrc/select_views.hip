// aura_select_views: Sec. 3.2.2, view importance-based filtering.
//
// For every visible (point, view) pair (Eq. 1, the shared fp32 decision functions):
//     S_dist = 1 / (1 + z),   S_angle = max(0, v . (-n)),   S_total = S_dist * S_angle,
// z the depth of the point in the camera frame, v the unit vector from the camera centre to the point, n the
// point's unit normal.  The k visible views with the largest S_total are kept, of equal scores the lower view
// index first.
//
// One thread per point, looping over the views of the point's object (camera rows by wave-uniform scalar reads,
// one depth texel per pair), the k best so far in registers.  The ray is taken in the camera frame, where it is
// Xc = R x + t itself: v . n = Xc . (R n) / |Xc|.  Traffic: 24 B per point in, 8 k + mask_pitch + 4 B out.
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

struct SelArgs {
  VisArgs vis;
  const float* xyz;
  const float* normals;
  int k;
  int* sel_view;       // [N][k]
  float* sel_score;    // [N][k] or nullptr
  uint8_t* sel_mask;   // [N][mask_pitch] or nullptr
  int mask_pitch;
  int* n_sel;          // [N] or nullptr
};

__global__ __launch_bounds__(256) void k_select_views(SelArgs a, ObjTable tab) {
  const ObjRange ob = tab.o[blockIdx.y];
  const int li = blockIdx.x * blockDim.x + threadIdx.x;
  if (li >= ob.n_pts) return;
  const long long i = ob.pt_begin + li;
  const float x = a.xyz[3 * i], y = a.xyz[3 * i + 1], z = a.xyz[3 * i + 2];
  const float nx = a.normals[3 * i], ny = a.normals[3 * i + 1], nz = a.normals[3 * i + 2];
  float best_s[kSelectMaxK];
  int best_v[kSelectMaxK];
#pragma unroll
  for (int t = 0; t < kSelectMaxK; ++t) {
    best_s[t] = -1.0f;   // below every score of a visible view
    best_v[t] = -1;
  }
  int seen = 0;
  for (int j = 0; j < ob.n_views; ++j) {
    const int v = ob.view_begin + j;
    const float* __restrict__ c = a.vis.cam + (long long)v * 16;
    const Proj p = project(c, x, y, z);
    const float* dv = a.vis.depth ? a.vis.depth + (long long)v * a.vis.H * a.vis.W : nullptr;
    if (!visible(a.vis, dv, p)) continue;
    ++seen;
    const float xc = __builtin_fmaf(c[2], z, __builtin_fmaf(c[1], y, __builtin_fmaf(c[0], x, c[9])));
    const float yc = __builtin_fmaf(c[5], z, __builtin_fmaf(c[4], y, __builtin_fmaf(c[3], x, c[10])));
    const float zc = p.z;
    const float rnx = c[0] * nx + c[1] * ny + c[2] * nz;   // the normal in the camera frame
    const float rny = c[3] * nx + c[4] * ny + c[5] * nz;
    const float rnz = c[6] * nx + c[7] * ny + c[8] * nz;
    const float len = sqrtf(xc * xc + yc * yc + zc * zc);
    const float s_angle = fmaxf(0.0f, -(xc * rnx + yc * rny + zc * rnz) / len);
    float s = s_angle / (1.0f + zc);
    int sv = j;
    // insert into the sorted list: a later view only moves ahead of an entry with a strictly smaller score; from
    // there on every entry moves down one place
    bool moving = false;
#pragma unroll
    for (int t = 0; t < kSelectMaxK; ++t) {
      moving = moving || s > best_s[t];
      if (t < a.k && moving) {
        const float ts = best_s[t];
        const int tv = best_v[t];
        best_s[t] = s;
        best_v[t] = sv;
        s = ts;
        sv = tv;
      }
    }
  }
#pragma unroll
  for (int t = 0; t < kSelectMaxK; ++t) {
    if (t < a.k) {
      a.sel_view[i * a.k + t] = best_v[t];
      if (a.sel_score) a.sel_score[i * a.k + t] = best_v[t] >= 0 ? best_s[t] : 0.0f;
    }
  }
  if (a.n_sel) a.n_sel[i] = seen < a.k ? seen : a.k;
  if (a.sel_mask) {
    uint8_t* __restrict__ row = a.sel_mask + i * a.mask_pitch;
    for (int j = 0; j < a.mask_pitch; ++j) {
      bool kept = false;
#pragma unroll
      for (int t = 0; t < kSelectMaxK; ++t) kept = kept || (t < a.k && best_v[t] == j);
      row[j] = kept ? 1 : 0;
    }
  }
}

hipError_t launch_select_views(const VisArgs& vis, const float* xyz, const float* normals, int k, int* sel_view,
                               float* sel_score, uint8_t* sel_mask, int mask_pitch, int* n_sel, const ObjTable& tab,
                               int n_obj, int max_pts, hipStream_t stream) {
  if (n_obj == 0 || max_pts == 0) return hipSuccess;
  SelArgs a{vis, xyz, normals, k, sel_view, sel_score, sel_mask, mask_pitch, n_sel};
  const dim3 grid((max_pts + 255) / 256, n_obj), block(256);
  hipLaunchKernelGGL(k_select_views, grid, block, 0, stream, a, tab);
  return hipGetLastError();
}

}  // namespace aura
