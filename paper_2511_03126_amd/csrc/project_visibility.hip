// aura_project_visibility: Sec. 3.1 "Visibility Checking", Eq. 1.
//
// One thread per point, looping over the views of the point's object.  Camera rows are read
// with a wave-uniform index (scalar loads); the only divergent access is the one depth texel per
// (point, view).  Traffic: 12 B per point in, vis_pitch + 4 B per point out, plus one 4-byte
// depth gather per pair, so the kernel is a small fraction of the fusion pass.
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

struct PvArgs {
  VisArgs vis;
  const float* xyz;
  uint8_t* out_vis;
  int* out_count;
  float* out_uvz;
  int vis_pitch;
  int words;      // rows of out_vis are 4-byte aligned: store four views per dword
};

__global__ __launch_bounds__(256) void k_project_visibility(PvArgs a, ObjTable tab) {
  const ObjRange ob = tab.o[blockIdx.y];
  int li = blockIdx.x * blockDim.x + threadIdx.x;
  if (li >= ob.n_pts) return;
  long long i = ob.pt_begin + li;
  float x = a.xyz[3 * i], y = a.xyz[3 * i + 1], z = a.xyz[3 * i + 2];
  uint8_t* row = a.out_vis + i * a.vis_pitch;
  int cnt = 0;
  const bool words = a.words != 0;
  uint32_t packed = 0;
  for (int j = 0; j < a.vis_pitch; ++j) {
    bool m = false;
    Proj p = {0.0f, 0.0f, 0.0f};
    if (j < ob.n_views) {
      int v = ob.view_begin + j;
      p = project(a.vis.cam + (long long)v * 16, x, y, z);
      const float* dv = a.vis.depth ? a.vis.depth + (long long)v * a.vis.H * a.vis.W : nullptr;
      m = visible(a.vis, dv, p);
    }
    cnt += m ? 1 : 0;
    if (words) {
      packed |= (m ? 1u : 0u) << (8 * (j & 3));
      if ((j & 3) == 3) {
        *reinterpret_cast<uint32_t*>(row + j - 3) = packed;
        packed = 0;
      }
    } else {
      row[j] = m ? 1 : 0;
    }
    if (a.out_uvz) {
      float* o = a.out_uvz + (i * a.vis_pitch + j) * 3;
      o[0] = p.u;
      o[1] = p.v;
      o[2] = p.z;
    }
  }
  if (a.out_count) a.out_count[i] = cnt;
}

hipError_t launch_project_visibility(const VisArgs& vis, const float* xyz, uint8_t* out_vis, int vis_pitch,
                                     int* out_count, float* out_uvz, const ObjTable& tab, int n_obj,
                                     int max_pts, hipStream_t stream) {
  if (n_obj == 0 || max_pts == 0) return hipSuccess;
  int words = ((vis_pitch & 3) == 0) && ((reinterpret_cast<uintptr_t>(out_vis) & 3) == 0);
  PvArgs a{vis, xyz, out_vis, out_count, out_uvz, vis_pitch, words};
  dim3 grid((max_pts + 255) / 256, n_obj), block(256);
  hipLaunchKernelGGL(k_project_visibility, grid, block, 0, stream, a, tab);
  return hipGetLastError();
}

}  // namespace aura
