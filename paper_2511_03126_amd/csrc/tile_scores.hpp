// Host-side interface of the scoring kernels that run on top of the matrix-core fusion path
// (tile_scores.hip), used by aura_fuse_scores.
#pragma once

#include "fuse_args.hpp"
#include "launch.hpp"

namespace aura {

struct TileScoreWs {
  float* factor;   // [N]: what the raw tile product of a point is multiplied by (1 / (count * norm), or 1 / count)
  uint32_t* G;     // [n_cells][Kpad]: similarity of every feature cell to every material, two 16-bit terms
  void* t_split;   // the text embeddings split into two 16-bit terms in operand order (written by launch_cell_scores)
  int Kpad;        // K rounded up to the matrix-core tile (32, 64 or 128)
};

size_t tile_scores_workspace_bytes(long long N, long long n_cells, int K);
TileScoreWs tile_scores_workspace(void* workspace, long long N, long long n_cells, int K);

// G = F . T^T over all n_cells cells (16-bit maps, D a multiple of 256).
hipError_t launch_cell_scores(const FeatArgs& feat, long long n_cells, const float* temb, int K, const TileScoreWs& ws,
                              hipStream_t stream);
// Scores, labels and properties of the objects of one launch table from the k-steps in `tws` (after the
// product kernel of the same table has run with ws.factor as its factor output).
hipError_t launch_tile_scores(const FeatArgs& feat, const TileWs& tws, const TileScoreWs& ws,
                              int K, const float* y, int P, float temperature, int unseen_zero, float* scores,
                              float* prop, int* label, const ObjTable& tab, int n_obj, int max_pts, hipStream_t stream);

}  // namespace aura
