// Kernel arguments shared by the fusion kernels (per-point gather, and the matrix-core tile path
// with its prepare and product kernels).
#pragma once

#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

// Scoring request to the tile path (Sec. 3.4.1): with the similarity of every feature cell to every material at hand
// (G, two 16-bit terms per value), the scores of a tile are one more small product over the tile's k-steps.
struct TileScoring {
  const uint32_t* G;    // [n_cells][Kpad]: hi | lo << 16
  int Kpad;             // K rounded up to the matrix-core tile
  int K, P;
  const float* temb;    // [K][D] fp32, for tiles without k-steps
  const float* y;       // [K][P], may be nullptr with prop
  float inv_T;
  int unseen_zero;      // properties of a point with all-zero similarities: 0 instead of the mean of y
  float* scores;        // [N][K]
  float* prop;          // [N][P] or nullptr
  int* label;           // [N] or nullptr
};

struct FuseArgs {
  VisArgs vis;
  FeatArgs feat;
  const float* xyz;
  float* fused;
  int* out_count;
  float norm_eps;
  int mean_only;
  float* out_factor;   // tile path only, may be nullptr: [N] factor applied to each point's raw tile product
  uint8_t* out_vis;    // tile path only, may be nullptr: [N][vis_pitch] visibility mask (Eq. 1), as aura_project_visibility
  int vis_pitch;
  const uint8_t* in_mask;   // may be nullptr: [N][in_mask_pitch], the views kept for each point (Sec. 3.2.2); given, it
  int in_mask_pitch;        // takes the place of the depth test (the caller passes no depth maps then)
  int two_kernels;          // tile path: keep the prepare and the product kernel apart (AURA_FUSE_TWO_KERNELS)
  TileScoring scoring;      // tile path: scores, labels and properties wanted along with the fused rows (G == nullptr: no)
};

// Whether view `local_view` (index within the object) takes part in the mean of point i.
__device__ __forceinline__ bool view_kept(const FuseArgs& a, long long i, int local_view) {
  return !a.in_mask || a.in_mask[i * a.in_mask_pitch + local_view] != 0;
}

// ---- workspace of the tile path ------------------------------------------------------------
// A tile is 32 consecutive points of one object.  The prepare kernel turns a tile into a list of
// k-steps; a k-step is 16 feature cells and the 32 x 16 matrix of bilinear weights of the tile's
// points for those cells, already in the register layout of the matrix-core A operand.

constexpr int kTilePts = 32;        // points per tile (M of the matrix-core product)
constexpr int kStepCells = 16;      // cells per k-step (K of the matrix-core product)

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

struct TileHdr {
  int nsteps;               // k-steps written for the tile; -1: the prepare kernel fused this tile itself
  int pad_[3];
  int cnt[kTilePts];        // views that see each point
};

struct __attribute__((aligned(64))) TileStep {
  uint32_t cell[kStepCells];   // byte offset of each cell row from the first feature element
  u32x4_t a_hi[64];            // lane l = 32 g + m: weights of point m for cells 8 g .. 8 g + 7 (16-bit)
  u32x4_t a_lo[64];            // second term of the two-term split of the same weights
};

struct TileWs {
  TileHdr* hdr;         // [n_tiles]
  unsigned* counters;   // [B][8]: tiles handed out so far, per object and XCD (zeroed by the prepare kernel)
  unsigned* status;     // one word per call, zero unless a kernel had something to report (see aura_fuse_status_offset)
  TileStep* steps;      // [n_tiles][quota]: every tile owns a fixed run of k-steps
  int quota;
  int obj_base;         // index of the launch's first object within the call
};

// Byte offset of a cell row as stored in a k-step (a multiple of 512 * units, units = D / 256 in 1..6) -> cell index.
__device__ __forceinline__ uint32_t cell_index(uint32_t off, uint32_t units) {
  const uint32_t q = off >> 9;
  switch (units) {
    case 1: return q;
    case 2: return q >> 1;
    case 3: return (uint32_t)(((unsigned long long)q * 0xAAAAAAABull) >> 33);
    case 4: return q >> 2;
    default: return (uint32_t)(((unsigned long long)(q >> 1) * 0xAAAAAAABull) >> 33);   // 6
  }
}

bool fuse_tile_supported(int dtype, int D, int Hf, int Wf, long long feat_bytes);
size_t fuse_tile_workspace_bytes(long long N, int B, int n_views);
size_t fuse_tile_status_offset(long long N, int B);   // byte offset of the status word within that workspace
// Splits a workspace of fuse_tile_workspace_bytes(N, B, n_views) bytes into its parts.
TileWs fuse_tile_workspace(void* workspace, long long N, int B, int n_views);
// ws.obj_base set.  *scored (may be nullptr) tells whether the launch also wrote what a.scoring asks for; if not, the
// k-steps and the factors are in the workspace for the scoring kernel.
hipError_t launch_fuse_tile(const FuseArgs& a, const TileWs& ws, const ObjTable& tab, int n_obj, int max_pts,
                            hipStream_t stream, bool* scored);

}  // namespace aura
