// Kernel arguments shared by the two fusion kernels (gather and matrix-core tile).
#pragma once

#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

struct FuseArgs {
  VisArgs vis;
  FeatArgs feat;
  const float* xyz;
  float* fused;
  int* out_count;
  float norm_eps;
  int mean_only;
};

bool fuse_tile_supported(int dtype, int D, int Hf, int Wf);
hipError_t launch_fuse_tile(const FuseArgs& a, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream);

}  // namespace aura
