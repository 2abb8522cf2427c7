// Host-side launch functions of the kernels (one per .hip file), called by the C ABI layer.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "aura_device.hpp"

namespace aura {

// Per-call description of the feature maps for the fusion kernel.
struct FeatArgs {
  const void* feat;   // [n_views][Hf][Wf][D]
  int Hf, Wf, D;
  int dtype;          // 0 fp32, 1 bf16, 2 fp16
  float pitch_x;      // W / Wf, H / Hf as fp32 quotients
  float pitch_y;
};

hipError_t launch_project_visibility(const VisArgs& vis, const float* xyz, uint8_t* out_vis, int vis_pitch,
                                     int* out_count, float* out_uvz, const ObjTable& tab, int n_obj,
                                     int max_pts, hipStream_t stream);

struct TileWs;
// tile_ws == nullptr: per-point gather kernel; otherwise the matrix-core tile path with that workspace.
struct TileScoring;
hipError_t launch_fuse_features(const VisArgs& vis, const FeatArgs& feat, const float* xyz, float* fused,
                                int* out_count, float norm_eps, int mean_only, const TileWs* tile_ws,
                                const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream,
                                float* out_factor = nullptr,    // tile path only: see FuseArgs::out_factor
                                uint8_t* out_vis = nullptr, int vis_pitch = 0,    // tile path only: see FuseArgs::out_vis
                                const uint8_t* in_mask = nullptr, int in_mask_pitch = 0,     // see FuseArgs::in_mask
                                int two_kernels = 0,                                        // see FuseArgs::two_kernels
                                const TileScoring* scoring = nullptr,    // tile path only: see FuseArgs::scoring
                                bool* scored = nullptr);                 // whether the launch did what `scoring` asks for

// Sec. 3.2.2, view importance-based filtering (select_views.hip).
constexpr int kSelectMaxK = 8;
hipError_t launch_select_views(const VisArgs& vis, const float* xyz, const float* normals, int k, int* sel_view,
                               float* sel_score, uint8_t* sel_mask, int mask_pitch, int* n_sel, const ObjTable& tab,
                               int n_obj, int max_pts, hipStream_t stream);

size_t scores_split_bytes(int D, int K);       // the split embeddings at the start of the scoring workspace
size_t scores_workspace_bytes(int D, int K);   // ... followed by room for an fp32 copy of 16-bit embeddings
hipError_t launch_widen_embeddings(const void* src, int dtype, long long n, float* dst, hipStream_t stream);
hipError_t launch_material_scores(const float* fused, long long N, int D, const float* temb, int K,
                                  const float* y, int P, float temperature, float* scores, float* prop,
                                  int* label, void* workspace, hipStream_t stream, int unseen_zero = 0);

// Objects of one integration launch (host side; copied into kernel arguments in chunks).
struct MassObj {
  long long pt_begin;
  int n_pts;
  float lo[3];
  float h;
};

size_t integrate_workspace_bytes(long long N, int B, int G);
hipError_t launch_property_integrate(const float* prop, int P, int p_index, const int* count, const float* vol,
                                     float vol_uniform, const MassObj* objs, int B, const float* xyz, int G,
                                     float* mass, long long* n_used, void* workspace, hipStream_t stream);

// Sec. 3.4.2, thickness-based integration and centre of mass (thickness_integrate.hip).
struct ThickObj {
  long long pt_begin;
  int n_pts;
  float box_len;   // characteristic length L of the object; < 0: longest side of its bounding box
};

bool thickness_supported(int K);
size_t thickness_workspace_bytes(long long N, int B);
hipError_t launch_thickness_integrate(const float* scores, int K, const float* y, int P, int p_index, const float* theta,
                                      const float* xyz, const int* count, const ThickObj* objs, int B, float temperature,
                                      float lambda, float scale_factor, float* zeta, float* total, float* com,
                                      float* b_adap, long long* n_used, void* workspace, hipStream_t stream);

// Sec. 3.2.1, adaptive voxel down-sampling (voxel_downsample.hip).
constexpr long long kVoxelMaxCells = 1ll << 24;   // cubes of all objects of a call, each object padded to 2048
struct VoxObj {
  long long pt_begin;
  int n_pts;
  float lo[3];
  float s;
  int dims[3];
};
bool voxel_grid(const float* lo, const float* hi, int n_target, float* s_out, int* dims);
long long voxel_padded_cells(long long cells);
size_t voxel_workspace_bytes(long long padded_cells);
hipError_t launch_voxel_downsample(const float* xyz, const VoxObj* objs, int B, float max_abs, long long n_points,
                                   float* out_xyz, int* out_count, long long capacity, int* out_offsets,
                                   int* voxel_of_point, void* workspace, hipStream_t stream);

// Sec. 3.2.3, multi-scale patches for the image encoder (patch_batch.hip).
bool patch_batch_supported(int L);
hipError_t launch_patch_batch(const float* cam, const uint8_t* images, int H, int W, const float* xyz, const int* sel_view,
                              int k, const float* scales, int L, int R, const float* mean, const float* inv_std,
                              void* out, bool half, uint8_t* valid, const ObjTable& tab, int n_obj, int max_pts,
                              hipStream_t stream);

// Sec. 3.2.2, normals of the sampled points (estimate_normals.hip).
struct NrmObj {
  long long pt_begin;
  int n_pts;
  int q_begin;
  int n_q;
  float centre[3];
};
hipError_t launch_estimate_normals(const float* xyz, const float* queries, const NrmObj* objs, int n_obj, int k,
                                   float* normals, float* evals, hipStream_t stream);

// Sec. 3.4.1 Eq. 5 (knn_densify.hip).
bool knn_supported(int Ns, int K, int k, int P);
size_t knn_workspace_bytes(int D, int Ns);
hipError_t launch_knn_densify(const float* fq, long long Nq, int D, const float* fs, int Ns, const float* ws, int K,
                              int k, const float* y, int P, float temperature, float* wq, float* prop, int* label,
                              int* nn_idx, void* workspace, hipStream_t stream);

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
hipError_t launch_calibration_fill(void* dst, size_t bytes, uint32_t value, hipStream_t stream);

}  // namespace aura
