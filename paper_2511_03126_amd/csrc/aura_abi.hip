// C ABI of libaura_fuse: argument validation and launch logic.  See include/aura_fuse.h for the
// contract of every entry point.  Validation happens before any HIP call, so every error path
// except AURA_ERR_HIP can be exercised on a machine without a GPU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <vector>

#include "../../include/aura_fuse.h"
#include "abi_util.hpp"
#include "fuse_args.hpp"
#include "launch.hpp"
#include "tile_scores.hpp"
#include "timing.hpp"

namespace {

thread_local int32_t g_last_hip_error = 0;
thread_local aura::TimingRequest g_timing;

using aura::aligned;
using aura::hip_status;

// Checks the object ranges and expands the "one object" shorthand.
aura_status_t check_objects(int64_t N, int32_t n_views, const int64_t* pt_offsets, const int32_t* view_offsets,
                            int32_t B, std::vector<aura::ObjRange>* out, int* max_views) {
  if (B < 1) return AURA_ERR_SHAPE;
  if ((pt_offsets == nullptr) != (view_offsets == nullptr)) return AURA_ERR_NULL;
  if (!pt_offsets && B != 1) return AURA_ERR_NULL;
  out->clear();
  *max_views = 0;
  int64_t tiles = 0;
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    const int64_t v0 = view_offsets ? view_offsets[b] : 0, v1 = view_offsets ? view_offsets[b + 1] : n_views;
    if (p1 < p0 || v1 < v0 || p0 < 0 || v0 < 0 || p1 > N || v1 > n_views) return AURA_ERR_SHAPE;
    if (p1 - p0 > 0x7fffffff) return AURA_ERR_SHAPE;
    if (b == 0 && (p0 != 0 || v0 != 0)) return AURA_ERR_SHAPE;
    if (b == B - 1 && (p1 != N || v1 != n_views)) return AURA_ERR_SHAPE;
    aura::ObjRange r{};
    r.pt_begin = p0;
    r.n_pts = (int)(p1 - p0);
    r.view_begin = (int)v0;
    r.n_views = (int)(v1 - v0);
    if (tiles > 0x7fffffff) return AURA_ERR_SHAPE;
    r.tile_begin = (int)tiles;
    tiles += (r.n_pts + aura::kTilePts - 1) / aura::kTilePts;
    out->push_back(r);
    *max_views = std::max(*max_views, r.n_views);
  }
  return AURA_OK;
}

aura_status_t check_views(const aura_views_t* v, const aura_params_t* p, bool need_feat) {
  if (!v || !p) return AURA_ERR_NULL;
  if (!v->cam) return AURA_ERR_NULL;
  if (!(p->flags & AURA_VIS_FRUSTUM_ONLY) && !v->depth) return AURA_ERR_NULL;
  if (v->n_views < 1 || v->H < 1 || v->W < 1) return AURA_ERR_SHAPE;
  if ((int64_t)v->H * v->W > 0x7fffffff) return AURA_ERR_SHAPE;
  if (need_feat) {
    if (!v->feat) return AURA_ERR_NULL;
    if (v->Hf < 1 || v->Wf < 1 || v->D < 1) return AURA_ERR_SHAPE;
    if ((int64_t)v->Hf * v->Wf * v->D > 0x7fffffff) return AURA_ERR_SHAPE;
    if ((int64_t)v->n_views * v->Hf * v->Wf > 0x7fffffff) return AURA_ERR_SHAPE;
    if (v->feat_dtype != AURA_F32 && v->feat_dtype != AURA_BF16 && v->feat_dtype != AURA_F16) return AURA_ERR_DTYPE;
    if (!aligned(v->feat, 16)) return AURA_ERR_ALIGN;
  }
  return AURA_OK;
}

aura::VisArgs vis_args(const aura_views_t* v, const aura_params_t* p) {
  aura::VisArgs a{};
  a.cam = v->cam;
  a.depth = (p->flags & AURA_VIS_FRUSTUM_ONLY) ? nullptr : v->depth;
  a.H = v->H;
  a.W = v->W;
  a.tau = p->tau;
  a.z_near = p->z_near;
  a.frustum_only = (p->flags & AURA_VIS_FRUSTUM_ONLY) ? 1 : 0;
  return a;
}

// Runs `launch(table, n_obj, max_pts)` over the objects in tables of kMaxObjPerLaunch.
template <typename F>
aura_status_t for_each_table(const std::vector<aura::ObjRange>& objs, F launch) {
  for (size_t base = 0; base < objs.size(); base += aura::kMaxObjPerLaunch) {
    aura::ObjTable tab{};
    const int n = (int)std::min<size_t>(aura::kMaxObjPerLaunch, objs.size() - base);
    int max_pts = 0;
    for (int t = 0; t < n; ++t) {
      tab.o[t] = objs[base + t];
      max_pts = std::max(max_pts, tab.o[t].n_pts);
    }
    aura_status_t s = hip_status(launch(tab, n, max_pts, (int)base));
    if (s != AURA_OK) return s;
  }
  return AURA_OK;
}

}  // namespace

aura_status_t aura::hip_status(hipError_t e) {
  if (e == hipSuccess) return AURA_OK;
  g_last_hip_error = (int32_t)e;
  return AURA_ERR_HIP;
}

aura::TimingRequest aura::take_timing_request() {
  const TimingRequest r = g_timing;
  g_timing = TimingRequest{};
  return r;
}

extern "C" {

int32_t aura_version(void) { return 200; }

const char* aura_strerror(aura_status_t status) {
  switch (status) {
    case AURA_OK: return "ok";
    case AURA_ERR_NULL: return "a required pointer is NULL";
    case AURA_ERR_SHAPE: return "a size is out of range or the object offsets are inconsistent";
    case AURA_ERR_DTYPE: return "unknown element type";
    case AURA_ERR_ALIGN: return "a pointer or row pitch is not aligned as documented";
    case AURA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case AURA_ERR_HIP: return "a HIP call failed (see aura_last_hip_error)";
    case AURA_ERR_UNSUPPORTED: return "request is valid but not supported by this build";
    default: return "unknown status";
  }
}

int32_t aura_last_hip_error(void) { return g_last_hip_error; }

// Whether aura_fuse_features takes the matrix-core tile path for these sizes.
static bool tile_path(int32_t dtype, int32_t D, int32_t Hf, int32_t Wf, int32_t n_views) {
  const long long feat_bytes = (long long)n_views * Hf * Wf * D * 2;
  return aura::fuse_tile_supported(dtype, D, Hf, Wf, feat_bytes);
}

static bool known_dtype(int32_t t) { return t == AURA_F32 || t == AURA_BF16 || t == AURA_F16; }

// Workspace of aura_fuse_scores: the fusion workspace, then (where the scores come from per-cell
// similarities) the factor and similarity arrays, then the workspace of aura_material_scores.  For
// aura_fuse_score_integrate (`single_pass`) the view counts and properties (for callers that do not want them), the
// workspace of the integration and, where the fused rows cannot be avoided, room for one chunk of them follow.
struct FuseScoresLayout {
  bool tile;        // fusion on the matrix cores
  bool by_cells;    // scores from per-cell similarities (needs tile and not too many cells)
  size_t fuse_off, cells_off, scores_off, total;
  size_t count_off, prop_off, mass_off, chunk_off;   // single pass only
  int64_t chunk_pts;                                  // points per chunk of fused rows
};

constexpr int64_t kChunkPts = 32768;   // aura_fuse_score_integrate without per-cell scores: fused rows live one chunk at a time

static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

static FuseScoresLayout fuse_scores_layout(int64_t N, int32_t B, int32_t n_views, int32_t Hf, int32_t Wf, int32_t D,
                                           int32_t dtype, int32_t K, bool single_pass = false, int32_t P = 0, int32_t G = 0) {
  FuseScoresLayout l{};
  const int64_t n_cells = (int64_t)n_views * Hf * Wf;
  l.tile = tile_path(dtype, D, Hf, Wf, n_views);
  // Per-cell similarities cost one pass over the maps; they pay when that is less than reading the fused rows back
  // (fewer cells than points), and without fused rows as long as the maps are not much larger than the rows would be.
  l.by_cells = l.tile && n_cells <= (single_pass ? 4 * N : N);
  if (single_pass && !l.by_cells) l.tile = false;   // chunks of rows from the gather kernel
  size_t off = 0;
  l.fuse_off = off;
  if (l.tile) off += round256(aura::fuse_tile_workspace_bytes(N, B, n_views));
  l.cells_off = off;
  if (l.by_cells) off += round256(aura::tile_scores_workspace_bytes(N, n_cells, K));
  l.scores_off = off;
  off += round256(aura::scores_workspace_bytes(D, K));
  if (single_pass) {
    l.count_off = off;
    off += round256((size_t)N * sizeof(int32_t));
    l.prop_off = off;
    off += round256((size_t)N * (size_t)P * sizeof(float));
    l.mass_off = off;
    off += round256(aura::integrate_workspace_bytes(N, B, G));
    l.chunk_off = off;
    l.chunk_pts = std::min<int64_t>(N, kChunkPts);   // also with per-cell scores: AURA_FUSE_GATHER switches them off
    off += round256((size_t)l.chunk_pts * (size_t)D * sizeof(float));
  }
  l.total = off;
  return l;
}

aura_status_t aura_workspace_bytes(int32_t call, const aura_sizes_t* sz, size_t* bytes) {
  if (!bytes || !sz) return AURA_ERR_NULL;
  *bytes = 0;
  if (call == AURA_CALL_MATERIAL_SCORES) {
    if (sz->D < 1 || sz->K < 1) return AURA_ERR_SHAPE;
    if (sz->K > 128) return AURA_ERR_UNSUPPORTED;
    *bytes = aura::scores_workspace_bytes(sz->D, sz->K);
    return AURA_OK;
  }
  if (call == AURA_CALL_PROPERTY_INTEGRATE) {
    if (sz->N < 0 || sz->B < 1 || sz->G < 0) return AURA_ERR_SHAPE;
    if (sz->B > 4096 || sz->G > 512 || (sz->G > 0 && (int64_t)sz->B * sz->G * sz->G * sz->G >= (1ll << 31)))
      return AURA_ERR_UNSUPPORTED;
    *bytes = aura::integrate_workspace_bytes(sz->N, sz->B, sz->G);
    return AURA_OK;
  }
  if (call == AURA_CALL_FUSE_FEATURES) {
    if (sz->N < 0 || sz->B < 1 || sz->n_views < 1 || sz->Hf < 1 || sz->Wf < 1 || sz->D < 1) return AURA_ERR_SHAPE;
    if (sz->feat_dtype != AURA_F32 && sz->feat_dtype != AURA_BF16 && sz->feat_dtype != AURA_F16) return AURA_ERR_DTYPE;
    if (tile_path(sz->feat_dtype, sz->D, sz->Hf, sz->Wf, sz->n_views))
      *bytes = aura::fuse_tile_workspace_bytes(sz->N, sz->B, sz->n_views);
    return AURA_OK;
  }
  if (call == AURA_CALL_KNN_DENSIFY) {
    if (sz->D < 1 || sz->Ns < 1) return AURA_ERR_SHAPE;
    if (sz->Ns > 256) return AURA_ERR_UNSUPPORTED;
    *bytes = aura::knn_workspace_bytes(sz->D, sz->Ns);
    return AURA_OK;
  }
  if (call == AURA_CALL_THICKNESS_INTEGRATE) {
    if (sz->N < 0 || sz->B < 1) return AURA_ERR_SHAPE;
    if (sz->B > 4096) return AURA_ERR_UNSUPPORTED;
    *bytes = aura::thickness_workspace_bytes(sz->N, sz->B);
    return AURA_OK;
  }
  if (call == AURA_CALL_FUSE_SCORE_INTEGRATE) {
    if (sz->N < 0 || sz->B < 1 || sz->n_views < 1 || sz->Hf < 1 || sz->Wf < 1 || sz->D < 1 || sz->K < 1 || sz->P < 1 ||
        sz->G < 0)
      return AURA_ERR_SHAPE;
    if (sz->feat_dtype != AURA_F32 && sz->feat_dtype != AURA_BF16 && sz->feat_dtype != AURA_F16) return AURA_ERR_DTYPE;
    if (sz->K > 128 || sz->P > 8 || sz->B > 4096 || sz->G > 512 ||
        (sz->G > 0 && (int64_t)sz->B * sz->G * sz->G * sz->G >= (1ll << 31)))
      return AURA_ERR_UNSUPPORTED;
    *bytes = fuse_scores_layout(sz->N, sz->B, sz->n_views, sz->Hf, sz->Wf, sz->D, sz->feat_dtype, sz->K, true, sz->P, sz->G).total;
    return AURA_OK;
  }
  if (call == AURA_CALL_FUSE_SCORES) {
    if (sz->N < 0 || sz->B < 1 || sz->n_views < 1 || sz->Hf < 1 || sz->Wf < 1 || sz->D < 1 || sz->K < 1) return AURA_ERR_SHAPE;
    if (sz->feat_dtype != AURA_F32 && sz->feat_dtype != AURA_BF16 && sz->feat_dtype != AURA_F16) return AURA_ERR_DTYPE;
    if (sz->K > 128) return AURA_ERR_UNSUPPORTED;
    *bytes = fuse_scores_layout(sz->N, sz->B, sz->n_views, sz->Hf, sz->Wf, sz->D, sz->feat_dtype, sz->K).total;
    return AURA_OK;
  }
  return AURA_ERR_UNSUPPORTED;
}

aura_status_t aura_fuse_status_offset(int32_t call, const aura_sizes_t* sz, size_t* offset, int32_t* present) {
  if (!sz || !offset || !present) return AURA_ERR_NULL;
  *offset = 0;
  *present = 0;
  if (call != AURA_CALL_FUSE_FEATURES && call != AURA_CALL_FUSE_SCORES && call != AURA_CALL_FUSE_SCORE_INTEGRATE)
    return AURA_ERR_UNSUPPORTED;
  if (sz->N < 0 || sz->B < 1 || sz->n_views < 1 || sz->Hf < 1 || sz->Wf < 1 || sz->D < 1) return AURA_ERR_SHAPE;
  if (!known_dtype(sz->feat_dtype)) return AURA_ERR_DTYPE;
  bool tile = tile_path(sz->feat_dtype, sz->D, sz->Hf, sz->Wf, sz->n_views);
  if (call == AURA_CALL_FUSE_SCORE_INTEGRATE) {
    if (sz->K < 1) return AURA_ERR_SHAPE;
    tile = fuse_scores_layout(sz->N, sz->B, sz->n_views, sz->Hf, sz->Wf, sz->D, sz->feat_dtype, sz->K, true, sz->P, sz->G).tile;
  }
  if (!tile) return AURA_OK;   // the gather kernel has nothing to report
  *offset = aura::fuse_tile_status_offset(sz->N, sz->B);   // the fusion workspace comes first in every layout
  *present = 1;
  return AURA_OK;
}

aura_status_t aura_project_visibility(const aura_views_t* views, const aura_params_t* params,
                                      const float* xyz, int64_t N,
                                      const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                      uint8_t* vis, int32_t vis_pitch, int32_t* count, float* uvz,
                                      void* stream) {
  aura_status_t s = check_views(views, params, false);
  if (s != AURA_OK) return s;
  if (N < 0) return AURA_ERR_SHAPE;
  std::vector<aura::ObjRange> objs;
  int max_views = 0;
  s = check_objects(N, views->n_views, pt_offsets, view_offsets, B, &objs, &max_views);
  if (s != AURA_OK) return s;
  if (vis_pitch < max_views || vis_pitch < 1) return AURA_ERR_SHAPE;
  if (N == 0) return AURA_OK;
  if (!xyz || !vis) return AURA_ERR_NULL;
  const aura::VisArgs va = vis_args(views, params);
  return for_each_table(objs, [&](const aura::ObjTable& tab, int n, int max_pts, int obj_base) {
    return aura::launch_project_visibility(va, xyz, vis, vis_pitch, count, uvz, tab, n, max_pts,
                                           static_cast<hipStream_t>(stream));
  });
}

// aura_fuse_features and aura_fuse_selected: the same launches, the second with a given selection of views.
static aura_status_t fuse_features_impl(const aura_views_t* views, const aura_params_t* params, const float* xyz, int64_t N,
                                        const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                        const uint8_t* sel_mask, int32_t mask_pitch, float* fused, int32_t* count,
                                        void* workspace, size_t workspace_bytes, void* stream);

aura_status_t aura_fuse_features(const aura_views_t* views, const aura_params_t* params,
                                 const float* xyz, int64_t N,
                                 const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                 float* fused, int32_t* count,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  return fuse_features_impl(views, params, xyz, N, pt_offsets, view_offsets, B, nullptr, 0, fused, count, workspace,
                            workspace_bytes, stream);
}

static aura_status_t fuse_features_impl(const aura_views_t* views, const aura_params_t* params, const float* xyz, int64_t N,
                                        const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                        const uint8_t* sel_mask, int32_t mask_pitch, float* fused, int32_t* count,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  // with a given selection the depth maps are not read
  aura_params_t par_sel;
  if (sel_mask && params) {
    par_sel = *params;
    par_sel.flags |= AURA_VIS_FRUSTUM_ONLY;
    params = &par_sel;
  }
  aura_status_t s = check_views(views, params, true);
  if (s != AURA_OK) return s;
  if (N < 0) return AURA_ERR_SHAPE;
  std::vector<aura::ObjRange> objs;
  int max_views = 0;
  s = check_objects(N, views->n_views, pt_offsets, view_offsets, B, &objs, &max_views);
  if (s != AURA_OK) return s;
  if (sel_mask && mask_pitch < max_views) return AURA_ERR_SHAPE;
  if (N == 0) return AURA_OK;
  if (!xyz || !fused) return AURA_ERR_NULL;
  if (!aligned(fused, 16)) return AURA_ERR_ALIGN;
  const aura::VisArgs va = vis_args(views, params);
  aura::FeatArgs fa{};
  fa.feat = views->feat;
  fa.Hf = views->Hf;
  fa.Wf = views->Wf;
  fa.D = views->D;
  fa.dtype = views->feat_dtype;
  fa.pitch_x = (float)views->W / (float)views->Wf;
  fa.pitch_y = (float)views->H / (float)views->Hf;
  const int mean_only = (params->flags & AURA_FUSE_MEAN_ONLY) ? 1 : 0;
  const hipStream_t st = static_cast<hipStream_t>(stream);
  // matrix-core tile path: 16-bit maps, D a multiple of 256, a workspace, and not switched off
  aura::TileWs tws{};
  const bool tile = workspace && !(params->flags & AURA_FUSE_GATHER) &&
                    tile_path(views->feat_dtype, views->D, views->Hf, views->Wf, views->n_views);
  if (tile) {
    if (!aligned(workspace, 256) || workspace_bytes < aura::fuse_tile_workspace_bytes(N, B, views->n_views))
      return AURA_ERR_WORKSPACE;
    tws = aura::fuse_tile_workspace(workspace, N, B, views->n_views);
  }
  if (!tile && workspace && aligned(workspace, 256) &&
      tile_path(views->feat_dtype, views->D, views->Hf, views->Wf, views->n_views) &&
      workspace_bytes >= aura::fuse_tile_workspace_bytes(N, B, views->n_views)) {
    // AURA_FUSE_GATHER with the workspace of the matrix-core kernels: its status word still says "nothing to report"
    const aura_status_t sc = hip_status(aura::launch_calibration_fill(
        static_cast<char*>(workspace) + aura::fuse_tile_status_offset(N, B), 16, 0u, st));
    if (sc != AURA_OK) return sc;
  }
  return for_each_table(objs, [&](const aura::ObjTable& tab, int n, int max_pts, int obj_base) {
    tws.obj_base = obj_base;
    return aura::launch_fuse_features(va, fa, xyz, fused, count, params->norm_eps, mean_only, tile ? &tws : nullptr,
                                      tab, n, max_pts, st, nullptr, nullptr, 0, sel_mask, mask_pitch,
                                      (params->flags & AURA_FUSE_TWO_KERNELS) ? 1 : 0);
  });
}

aura_status_t aura_fuse_selected(const aura_views_t* views, const aura_params_t* params, const float* xyz, int64_t N,
                                 const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                 const uint8_t* sel_mask, int32_t mask_pitch, float* fused, int32_t* count,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (!views || !params) return AURA_ERR_NULL;
  if (N > 0 && !sel_mask) return AURA_ERR_NULL;
  return fuse_features_impl(views, params, xyz, N, pt_offsets, view_offsets, B, sel_mask, mask_pitch, fused, count,
                            workspace, workspace_bytes, stream);
}

aura_status_t aura_select_views(const aura_views_t* views, const aura_params_t* params, const float* xyz,
                                const float* normals, int64_t N, const int64_t* pt_offsets,
                                const int32_t* view_offsets, int32_t B, int32_t k, int32_t* sel_view, float* sel_score,
                                uint8_t* sel_mask, int32_t mask_pitch, int32_t* n_sel, void* stream) {
  aura_status_t s = check_views(views, params, false);
  if (s != AURA_OK) return s;
  if (N < 0 || k < 1) return AURA_ERR_SHAPE;
  if (k > aura::kSelectMaxK) return AURA_ERR_UNSUPPORTED;
  std::vector<aura::ObjRange> objs;
  int max_views = 0;
  s = check_objects(N, views->n_views, pt_offsets, view_offsets, B, &objs, &max_views);
  if (s != AURA_OK) return s;
  if (sel_mask && mask_pitch < max_views) return AURA_ERR_SHAPE;
  if (N == 0) return AURA_OK;
  if (!xyz || !normals || !sel_view) return AURA_ERR_NULL;
  const aura::VisArgs va = vis_args(views, params);
  const hipStream_t st = static_cast<hipStream_t>(stream);
  return for_each_table(objs, [&](const aura::ObjTable& tab, int n, int max_pts, int) {
    return aura::launch_select_views(va, xyz, normals, k, sel_view, sel_score, sel_mask, mask_pitch, n_sel, tab, n,
                                     max_pts, st);
  });
}

// The text embeddings as fp32: as given, or (bf16 / fp16) widened into the copy area of a scoring workspace.
static aura_status_t embeddings_f32(const void* temb, int32_t temb_dtype, int32_t K, int32_t D, char* scores_ws,
                                    hipStream_t st, const float** out) {
  if (temb_dtype == AURA_F32) {
    *out = static_cast<const float*>(temb);
    return AURA_OK;
  }
  float* copy = reinterpret_cast<float*>(scores_ws + aura::scores_split_bytes(D, K));
  *out = copy;
  return hip_status(aura::launch_widen_embeddings(temb, temb_dtype, (long long)K * D, copy, st));
}

// What aura_fuse_scores and aura_fuse_score_integrate share: the checks (everything except the workspace and the
// outputs that only one of them has), then the launches.
static aura_status_t check_fuse_scores(const aura_views_t* views, const aura_params_t* params, int64_t N,
                                       const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B, const void* temb,
                                       int32_t temb_dtype, int32_t K, const float* y, int32_t P, const float* prop,
                                       const uint8_t* vis, int32_t vis_pitch, std::vector<aura::ObjRange>* objs) {
  aura_status_t s = check_views(views, params, true);
  if (s != AURA_OK) return s;
  if (!temb) return AURA_ERR_NULL;
  if (N < 0 || K < 1 || P < 0) return AURA_ERR_SHAPE;
  if (!known_dtype(temb_dtype)) return AURA_ERR_DTYPE;
  if (prop && (!y || P < 1)) return AURA_ERR_NULL;
  if (!(params->temperature > 0.0f)) return AURA_ERR_SHAPE;
  if (K > 128 || P > 8) return AURA_ERR_UNSUPPORTED;
  int max_views = 0;
  s = check_objects(N, views->n_views, pt_offsets, view_offsets, B, objs, &max_views);
  if (s != AURA_OK) return s;
  if (vis && (vis_pitch < max_views || vis_pitch < 1)) return AURA_ERR_SHAPE;
  return AURA_OK;
}

// fused == nullptr (aura_fuse_score_integrate): no [N][D] array exists.  With per-cell scores the fusion kernels simply
// do not store their rows; otherwise the rows of lay.chunk_pts points at a time go through the chunk buffer in the
// workspace (small enough to stay in the last-level cache between the fusion and the scoring kernel).
static aura_status_t run_fuse_scores(const aura_views_t* views, const aura_params_t* params, const float* xyz, int64_t N,
                                     int32_t B, const std::vector<aura::ObjRange>& objs, const void* temb,
                                     int32_t temb_dtype, int32_t K,
                                     const float* y, int32_t P, float* fused, int32_t* count, uint8_t* vis,
                                     int32_t vis_pitch, float* scores, float* prop, int32_t* label, FuseScoresLayout lay,
                                     char* wbase, hipStream_t st) {
  if ((params->flags & AURA_FUSE_GATHER) && lay.tile) {
    // the matrix-core kernels stay out: the status word in their part of the workspace still says "nothing to report"
    const aura_status_t sc = hip_status(aura::launch_calibration_fill(
        wbase + lay.fuse_off + aura::fuse_tile_status_offset(N, B), 16, 0u, st));
    if (sc != AURA_OK) return sc;
    lay.tile = lay.by_cells = false;
  }
  const aura::VisArgs va = vis_args(views, params);
  aura::FeatArgs fa{};
  fa.feat = views->feat;
  fa.Hf = views->Hf;
  fa.Wf = views->Wf;
  fa.D = views->D;
  fa.dtype = views->feat_dtype;
  fa.pitch_x = (float)views->W / (float)views->Wf;
  fa.pitch_y = (float)views->H / (float)views->Hf;
  const int mean_only = (params->flags & AURA_FUSE_MEAN_ONLY) ? 1 : 0;
  const int64_t n_cells = (int64_t)views->n_views * views->Hf * views->Wf;
  const int unseen_zero = (params->flags & AURA_UNSEEN_ZERO) ? 1 : 0;
  const float* t32 = nullptr;
  aura_status_t s = embeddings_f32(temb, temb_dtype, K, views->D, wbase + lay.scores_off, st, &t32);
  if (s != AURA_OK) return s;

  if (!fused && !lay.by_cells) {
    float* chunk = reinterpret_cast<float*>(wbase + lay.chunk_off);
    std::vector<aura::ObjRange> part;
    for (int64_t c0 = 0; c0 < N; c0 += lay.chunk_pts) {
      const int64_t c1 = std::min(N, c0 + lay.chunk_pts);
      part.clear();
      for (const aura::ObjRange& o : objs) {
        const int64_t p0 = std::max<int64_t>(o.pt_begin, c0), p1 = std::min<int64_t>(o.pt_begin + o.n_pts, c1);
        if (p1 <= p0) continue;
        aura::ObjRange r = o;
        r.pt_begin = p0;
        r.n_pts = (int)(p1 - p0);
        r.tile_begin = 0;
        part.push_back(r);
      }
      // the kernels index rows by absolute point number: row c0 is the chunk's first
      float* rows = reinterpret_cast<float*>(reinterpret_cast<uintptr_t>(chunk) - (uintptr_t)c0 * (uintptr_t)views->D * sizeof(float));
      s = for_each_table(part, [&](const aura::ObjTable& tab, int n, int max_pts, int) {
        hipError_t e = hipSuccess;
        if (vis) e = aura::launch_project_visibility(va, xyz, vis, vis_pitch, nullptr, nullptr, tab, n, max_pts, st);
        if (e != hipSuccess) return e;
        return aura::launch_fuse_features(va, fa, xyz, rows, count, params->norm_eps, mean_only, nullptr, tab, n, max_pts, st);
      });
      if (s != AURA_OK) return s;
      s = hip_status(aura::launch_material_scores(chunk, c1 - c0, views->D, t32, K, y, P, params->temperature,
                                                  scores + c0 * K, prop ? prop + c0 * P : nullptr,
                                                  label ? label + c0 : nullptr, wbase + lay.scores_off, st, unseen_zero));
      if (s != AURA_OK) return s;
    }
    return AURA_OK;
  }

  aura::TileWs tws{};
  aura::TileScoreWs sws{};
  if (lay.tile) tws = aura::fuse_tile_workspace(wbase + lay.fuse_off, N, B, views->n_views);
  if (lay.by_cells) {
    sws = aura::tile_scores_workspace(wbase + lay.cells_off, N, n_cells, K);
    s = hip_status(aura::launch_cell_scores(fa, n_cells, t32, K, sws, st));
    if (s != AURA_OK) return s;
  }
  s = for_each_table(objs, [&](const aura::ObjTable& tab, int n, int max_pts, int obj_base) {
    tws.obj_base = obj_base;
    hipError_t e = hipSuccess;
    if (vis && !lay.tile)   // the gather kernel does not write the mask: the visibility kernel does
      e = aura::launch_project_visibility(va, xyz, vis, vis_pitch, nullptr, nullptr, tab, n, max_pts, st);
    if (e != hipSuccess) return e;
    const aura::TileScoring want{sws.G, sws.Kpad, K, P, t32, y, 1.0f / params->temperature, unseen_zero, scores, prop, label};
    bool scored = false;   // the one-kernel form of the fusion scores its tiles itself where it can
    e = aura::launch_fuse_features(va, fa, xyz, fused, count, params->norm_eps, mean_only,
                                   lay.tile ? &tws : nullptr, tab, n, max_pts, st, lay.by_cells ? sws.factor : nullptr,
                                   vis, vis_pitch, nullptr, 0, (params->flags & AURA_FUSE_TWO_KERNELS) ? 1 : 0,
                                   lay.by_cells ? &want : nullptr, &scored);
    if (e != hipSuccess || !lay.by_cells || scored) return e;
    return aura::launch_tile_scores(fa, tws, sws, K, y, P, params->temperature, unseen_zero, scores, prop, label, tab, n,
                                    max_pts, st);
  });
  if (s != AURA_OK || lay.by_cells) return s;
  return hip_status(aura::launch_material_scores(fused, N, views->D, t32, K, y, P, params->temperature, scores, prop,
                                                 label, wbase + lay.scores_off, st, unseen_zero));
}

aura_status_t aura_fuse_scores(const aura_views_t* views, const aura_params_t* params,
                               const float* xyz, int64_t N,
                               const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                               const void* temb, int32_t temb_dtype, int32_t K, const float* y, int32_t P,
                               float* fused, int32_t* count, uint8_t* vis, int32_t vis_pitch,
                               float* scores, float* prop, int32_t* label,
                               void* workspace, size_t workspace_bytes, void* stream) {
  std::vector<aura::ObjRange> objs;
  aura_status_t s = check_fuse_scores(views, params, N, pt_offsets, view_offsets, B, temb, temb_dtype, K, y, P, prop, vis,
                                      vis_pitch, &objs);
  if (s != AURA_OK) return s;
  if (N == 0) return AURA_OK;
  if (!xyz || !fused || !scores) return AURA_ERR_NULL;
  if (!aligned(fused, 16)) return AURA_ERR_ALIGN;
  const FuseScoresLayout lay = fuse_scores_layout(N, B, views->n_views, views->Hf, views->Wf, views->D, views->feat_dtype, K);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < lay.total) return AURA_ERR_WORKSPACE;
  return run_fuse_scores(views, params, xyz, N, B, objs, temb, temb_dtype, K, y, P, fused, count, vis, vis_pitch, scores,
                         prop, label, lay, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

// Checks the objects of an integration and fills their launch records.
static aura_status_t mass_objects(int64_t N, const int64_t* pt_offsets, int32_t B, const float* grid_lo, const float* grid_h,
                                  int32_t G, std::vector<aura::MassObj>* objs) {
  objs->assign((size_t)B, aura::MassObj{});
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    if (p1 < p0 || p0 < 0 || p1 > N || p1 - p0 > 0x7fffffff) return AURA_ERR_SHAPE;
    if ((b == 0 && p0 != 0) || (b == B - 1 && p1 != N)) return AURA_ERR_SHAPE;
    aura::MassObj& o = (*objs)[(size_t)b];
    o.pt_begin = p0;
    o.n_pts = (int)(p1 - p0);
    o.lo[0] = o.lo[1] = o.lo[2] = 0.0f;
    o.h = 1.0f;
    if (G > 0) {
      o.lo[0] = grid_lo[3 * b];
      o.lo[1] = grid_lo[3 * b + 1];
      o.lo[2] = grid_lo[3 * b + 2];
      o.h = grid_h[b];
      if (!(o.h > 0.0f)) return AURA_ERR_SHAPE;
    }
  }
  return AURA_OK;
}

aura_status_t aura_fuse_score_integrate(const aura_views_t* views, const aura_params_t* params,
                                        const float* xyz, int64_t N,
                                        const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                        const void* temb, int32_t temb_dtype, int32_t K, const float* y, int32_t P,
                                        int32_t p_index, const float* vol, float vol_uniform,
                                        const float* grid_lo, const float* grid_h, int32_t G,
                                        int32_t* count, uint8_t* vis, int32_t vis_pitch,
                                        float* scores, float* prop, int32_t* label,
                                        float* mass, int64_t* n_used,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  std::vector<aura::ObjRange> objs;
  aura_status_t s = check_fuse_scores(views, params, N, pt_offsets, view_offsets, B, temb, temb_dtype, K, y, P, nullptr, vis,
                                      vis_pitch, &objs);
  if (s != AURA_OK) return s;
  if (!y || !mass) return AURA_ERR_NULL;
  if (P < 1 || p_index < 0 || p_index >= P || G < 0) return AURA_ERR_SHAPE;
  if (G > 0 && (!grid_lo || !grid_h)) return AURA_ERR_NULL;
  if (B > 4096 || G > 512 || (G > 0 && (int64_t)B * G * G * G >= (1ll << 31))) return AURA_ERR_UNSUPPORTED;
  std::vector<aura::MassObj> mobjs;
  s = mass_objects(N, pt_offsets, B, grid_lo, grid_h, G, &mobjs);
  if (s != AURA_OK) return s;
  if (N > 0 && (!xyz || !scores)) return AURA_ERR_NULL;
  const FuseScoresLayout lay = fuse_scores_layout(N, B, views->n_views, views->Hf, views->Wf, views->D, views->feat_dtype, K,
                                                  true, P, G);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < lay.total) return AURA_ERR_WORKSPACE;
  char* wbase = static_cast<char*>(workspace);
  const hipStream_t st = static_cast<hipStream_t>(stream);
  if (!count) count = reinterpret_cast<int32_t*>(wbase + lay.count_off);
  if (!prop) prop = reinterpret_cast<float*>(wbase + lay.prop_off);
  if (N > 0) {
    s = run_fuse_scores(views, params, xyz, N, B, objs, temb, temb_dtype, K, y, P, nullptr, count, vis, vis_pitch, scores,
                        prop, label, lay, wbase, st);
    if (s != AURA_OK) return s;
  }
  return hip_status(aura::launch_property_integrate(prop, P, p_index, count, vol, vol_uniform, mobjs.data(), B, xyz, G, mass,
                                                    reinterpret_cast<long long*>(n_used), wbase + lay.mass_off, st));
}

aura_status_t aura_material_scores(const float* fused, int64_t N, int32_t D,
                                   const void* temb, int32_t temb_dtype, int32_t K,
                                   const float* y, int32_t P, const aura_params_t* params,
                                   float* scores, float* prop, int32_t* label,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  if (!params || !temb) return AURA_ERR_NULL;
  if (N < 0 || D < 1 || K < 1 || P < 0) return AURA_ERR_SHAPE;
  if (!known_dtype(temb_dtype)) return AURA_ERR_DTYPE;
  if (prop && (!y || P < 1)) return AURA_ERR_NULL;
  if (!(params->temperature > 0.0f)) return AURA_ERR_SHAPE;
  if (K > 128 || P > 8) return AURA_ERR_UNSUPPORTED;
  if (N == 0) return AURA_OK;
  if (!fused || !scores) return AURA_ERR_NULL;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < aura::scores_workspace_bytes(D, K))
    return AURA_ERR_WORKSPACE;
  const hipStream_t st = static_cast<hipStream_t>(stream);
  const float* t32 = nullptr;
  const aura_status_t s = embeddings_f32(temb, temb_dtype, K, D, static_cast<char*>(workspace), st, &t32);
  if (s != AURA_OK) return s;
  return hip_status(aura::launch_material_scores(fused, N, D, t32, K, y, P, params->temperature, scores, prop, label,
                                                 workspace, st, (params->flags & AURA_UNSEEN_ZERO) ? 1 : 0));
}

aura_status_t aura_knn_densify(const float* fq, int64_t Nq, int32_t D, const float* fs, int32_t Ns,
                               const float* ws, int32_t K, int32_t k, const float* y, int32_t P,
                               const aura_params_t* params, float* wq, float* prop, int32_t* label,
                               int32_t* nn_idx, void* workspace, size_t workspace_bytes, void* stream) {
  if (!params || !fs || !ws) return AURA_ERR_NULL;
  if (Nq < 0 || D < 1 || Ns < 1 || K < 1 || k < 1 || P < 0) return AURA_ERR_SHAPE;
  if (prop && (!y || P < 1)) return AURA_ERR_NULL;
  if (!(params->temperature > 0.0f)) return AURA_ERR_SHAPE;
  if (!aura::knn_supported(Ns, K, k, P)) return AURA_ERR_UNSUPPORTED;
  if (Nq == 0) return AURA_OK;
  if (!fq || !wq) return AURA_ERR_NULL;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < aura::knn_workspace_bytes(D, Ns)) return AURA_ERR_WORKSPACE;
  return hip_status(aura::launch_knn_densify(fq, Nq, D, fs, Ns, ws, K, k, y, P, params->temperature, wq, prop, label,
                                             nn_idx, workspace, static_cast<hipStream_t>(stream)));
}

aura_status_t aura_property_integrate(const float* prop, int64_t N, int32_t P, int32_t p_index,
                                      const int32_t* count, const float* vol, float vol_uniform,
                                      const int64_t* pt_offsets, int32_t B,
                                      const float* xyz, const float* grid_lo, const float* grid_h, int32_t G,
                                      float* mass, int64_t* n_used,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  if (N < 0 || P < 1 || p_index < 0 || p_index >= P || B < 1 || G < 0) return AURA_ERR_SHAPE;
  if (!pt_offsets && B != 1) return AURA_ERR_NULL;
  if (!mass) return AURA_ERR_NULL;
  if (G > 0 && (!grid_lo || !grid_h)) return AURA_ERR_NULL;
  if (B > 4096 || G > 512 || (G > 0 && (int64_t)B * G * G * G >= (1ll << 31))) return AURA_ERR_UNSUPPORTED;
  std::vector<aura::MassObj> objs;
  const aura_status_t so = mass_objects(N, pt_offsets, B, grid_lo, grid_h, G, &objs);
  if (so != AURA_OK) return so;
  if (N > 0 && (!prop || (G > 0 && !xyz))) return AURA_ERR_NULL;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < aura::integrate_workspace_bytes(N, B, G))
    return AURA_ERR_WORKSPACE;
  return hip_status(aura::launch_property_integrate(prop, P, p_index, count, vol, vol_uniform, objs.data(), B, xyz, G,
                                                    mass, reinterpret_cast<long long*>(n_used), workspace,
                                                    static_cast<hipStream_t>(stream)));
}

aura_status_t aura_thickness_integrate(const float* scores, int64_t N, int32_t K, const float* y, int32_t P, int32_t p_index,
                                       const float* theta, const float* xyz, const int32_t* count,
                                       const int64_t* pt_offsets, int32_t B, const float* box_len,
                                       const aura_params_t* params, float lambda, float scale_factor,
                                       float* zeta, float* total, float* com, float* b_adap, int64_t* n_used,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!params || !total) return AURA_ERR_NULL;
  if (N < 0 || K < 1 || P < 1 || p_index < 0 || p_index >= P || B < 1) return AURA_ERR_SHAPE;
  if (!(params->temperature > 0.0f) || !(lambda == lambda) || !(scale_factor >= 0.0f)) return AURA_ERR_SHAPE;
  if (!pt_offsets && B != 1) return AURA_ERR_NULL;
  if (B > 4096 || !aura::thickness_supported(K)) return AURA_ERR_UNSUPPORTED;
  std::vector<aura::ThickObj> objs((size_t)B);
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    if (p1 < p0 || p0 < 0 || p1 > N || p1 - p0 > 0x7fffffff) return AURA_ERR_SHAPE;
    if ((b == 0 && p0 != 0) || (b == B - 1 && p1 != N)) return AURA_ERR_SHAPE;
    aura::ThickObj& o = objs[(size_t)b];
    o.pt_begin = p0;
    o.n_pts = (int)(p1 - p0);
    o.box_len = -1.0f;
    if (box_len) {
      if (!(box_len[b] >= 0.0f)) return AURA_ERR_SHAPE;
      o.box_len = box_len[b];
    }
  }
  if (N > 0 && (!scores || !y || !theta || !xyz)) return AURA_ERR_NULL;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < aura::thickness_workspace_bytes(N, B))
    return AURA_ERR_WORKSPACE;
  return hip_status(aura::launch_thickness_integrate(scores, K, y, P, p_index, theta, xyz, count, objs.data(), B,
                                                     params->temperature, lambda, scale_factor, zeta, total, com, b_adap,
                                                     reinterpret_cast<long long*>(n_used), workspace,
                                                     static_cast<hipStream_t>(stream)));
}

aura_status_t aura_estimate_normals(const float* xyz, int64_t N, const int64_t* pt_offsets, const float* queries, int64_t M,
                                    const int64_t* q_offsets, int32_t B, const float* centre, int32_t k, float* normals,
                                    float* evals, void* stream) {
  if (N < 0 || M < 0 || B < 1 || k < 1) return AURA_ERR_SHAPE;
  if ((pt_offsets == nullptr) != (q_offsets == nullptr)) return AURA_ERR_NULL;
  if (!pt_offsets && B != 1) return AURA_ERR_NULL;
  if (!centre) return AURA_ERR_NULL;
  if (B > 4096) return AURA_ERR_UNSUPPORTED;
  std::vector<aura::NrmObj> objs((size_t)B);
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    const int64_t q0 = q_offsets ? q_offsets[b] : 0, q1 = q_offsets ? q_offsets[b + 1] : M;
    if (p1 < p0 || q1 < q0 || p0 < 0 || q0 < 0 || p1 > N || q1 > M) return AURA_ERR_SHAPE;
    if (p1 - p0 > 0x7fffffff || q1 > 0x7fffffff) return AURA_ERR_SHAPE;
    if (b == 0 && (p0 != 0 || q0 != 0)) return AURA_ERR_SHAPE;
    if (b == B - 1 && (p1 != N || q1 != M)) return AURA_ERR_SHAPE;
    aura::NrmObj& o = objs[(size_t)b];
    o.pt_begin = p0; o.n_pts = (int)(p1 - p0); o.q_begin = (int)q0; o.n_q = (int)(q1 - q0);
    for (int c = 0; c < 3; ++c) {
      if (!(centre[3 * b + c] == centre[3 * b + c])) return AURA_ERR_SHAPE;
      o.centre[c] = centre[3 * b + c];
    }
  }
  if (M == 0) return AURA_OK;
  if (!queries || !normals || (N > 0 && !xyz)) return AURA_ERR_NULL;
  for (int base = 0; base < B; base += aura::kMaxObjPerLaunch) {
    const int n = std::min(aura::kMaxObjPerLaunch, B - base);
    const aura_status_t s = hip_status(aura::launch_estimate_normals(xyz, queries, objs.data() + base, n, k, normals, evals,
                                                                     static_cast<hipStream_t>(stream)));
    if (s != AURA_OK) return s;
  }
  return AURA_OK;
}

aura_status_t aura_patch_batch(const float* cam, int32_t n_views, int32_t H, int32_t W, const uint8_t* images,
                               const float* xyz, int64_t M, const int64_t* pt_offsets, const int32_t* view_offsets,
                               int32_t B, const int32_t* sel_view, int32_t k, const float* scales, int32_t L, int32_t R,
                               const float* mean, const float* inv_std, void* out, int32_t out_dtype, uint8_t* valid,
                               void* stream) {
  if (M < 0 || n_views < 1 || H < 1 || W < 1 || k < 1 || L < 1 || R < 1) return AURA_ERR_SHAPE;
  if ((int64_t)H * W * 3 > 0x7fffffff) return AURA_ERR_SHAPE;
  if (out_dtype != AURA_F32 && out_dtype != AURA_F16) return out_dtype == AURA_BF16 ? AURA_ERR_UNSUPPORTED : AURA_ERR_DTYPE;
  if (!scales) return AURA_ERR_NULL;
  if (!aura::patch_batch_supported(L)) return AURA_ERR_UNSUPPORTED;
  for (int l = 0; l < L; ++l)
    if (!(scales[l] > 0.0f)) return AURA_ERR_SHAPE;
  if (inv_std)
    for (int c = 0; c < 3; ++c)
      if (!(inv_std[c] == inv_std[c])) return AURA_ERR_SHAPE;
  std::vector<aura::ObjRange> objs;
  int max_views = 0;
  const aura_status_t s = check_objects(M, n_views, pt_offsets, view_offsets, B, &objs, &max_views);
  if (s != AURA_OK) return s;
  if (M == 0) return AURA_OK;
  if (!cam || !images || !xyz || !sel_view || !out) return AURA_ERR_NULL;
  if (!aligned(out, out_dtype == AURA_F16 ? 2 : 4)) return AURA_ERR_ALIGN;
  for (const aura::ObjRange& o : objs)
    if ((int64_t)o.n_pts * k * L * ((R + 31) / 32) > 0x7fffffff) return AURA_ERR_UNSUPPORTED;   // one workgroup per 32 rows
  const hipStream_t st = static_cast<hipStream_t>(stream);
  return for_each_table(objs, [&](const aura::ObjTable& tab, int n, int max_pts, int) {
    return aura::launch_patch_batch(cam, images, H, W, xyz, sel_view, k, scales, L, R, mean, inv_std, out,
                                    out_dtype == AURA_F16, valid, tab, n, max_pts, st);
  });
}

aura_status_t aura_voxel_grid(const float* box_lo, const float* box_hi, int32_t n_target, float* s_voxel, int32_t* dims) {
  if (!box_lo || !box_hi || !s_voxel || !dims) return AURA_ERR_NULL;
  if (n_target < 1) return AURA_ERR_SHAPE;
  for (int a = 0; a < 3; ++a)
    if (!(box_hi[a] >= box_lo[a])) return AURA_ERR_SHAPE;
  int d[3];
  if (!aura::voxel_grid(box_lo, box_hi, n_target, s_voxel, d)) return AURA_ERR_UNSUPPORTED;
  dims[0] = d[0]; dims[1] = d[1]; dims[2] = d[2];
  return AURA_OK;
}

// Grids of the objects of a call; total = cubes of all objects, each object padded as the kernels lay them out.
static aura_status_t voxel_objects(const float* box_lo, const float* box_hi, int32_t B, int32_t n_target,
                                   std::vector<aura::VoxObj>* objs, long long* total, float* max_abs) {
  if (!box_lo || !box_hi) return AURA_ERR_NULL;
  if (B < 1 || n_target < 1) return AURA_ERR_SHAPE;
  if (B > aura::kMaxObjPerLaunch) return AURA_ERR_UNSUPPORTED;
  objs->assign((size_t)B, aura::VoxObj{});
  *total = 0;
  *max_abs = 0.0f;
  for (int b = 0; b < B; ++b) {
    aura::VoxObj& o = (*objs)[(size_t)b];
    for (int a = 0; a < 3; ++a) {
      const float lo = box_lo[3 * b + a], hi = box_hi[3 * b + a];
      if (!(hi >= lo)) return AURA_ERR_SHAPE;
      o.lo[a] = lo;
      // points up to one box extent outside the box still sum without overflow
      const float reach = std::max(std::fabs(lo - (hi - lo)), std::fabs(hi + (hi - lo)));
      *max_abs = std::max(*max_abs, reach);
    }
    if (!aura::voxel_grid(box_lo + 3 * b, box_hi + 3 * b, n_target, &o.s, o.dims)) return AURA_ERR_UNSUPPORTED;
    *total += aura::voxel_padded_cells((long long)o.dims[0] * o.dims[1] * o.dims[2]);
    if (*total > aura::kVoxelMaxCells) return AURA_ERR_UNSUPPORTED;
  }
  return AURA_OK;
}

aura_status_t aura_voxel_workspace_bytes(const float* box_lo, const float* box_hi, int32_t B, int32_t n_target,
                                         size_t* bytes) {
  if (!bytes) return AURA_ERR_NULL;
  *bytes = 0;
  std::vector<aura::VoxObj> objs;
  long long total = 0;
  float max_abs = 0.0f;
  const aura_status_t s = voxel_objects(box_lo, box_hi, B, n_target, &objs, &total, &max_abs);
  if (s != AURA_OK) return s;
  *bytes = aura::voxel_workspace_bytes(total);
  return AURA_OK;
}

aura_status_t aura_voxel_downsample(const float* xyz, int64_t N, const int64_t* pt_offsets, int32_t B,
                                    const float* box_lo, const float* box_hi, int32_t n_target, float* out_xyz,
                                    int32_t* out_count, int64_t out_capacity, int32_t* out_offsets,
                                    int32_t* voxel_of_point, void* workspace, size_t workspace_bytes, void* stream) {
  if (N < 0 || out_capacity < 0) return AURA_ERR_SHAPE;
  if (!pt_offsets && B != 1) return AURA_ERR_NULL;
  std::vector<aura::VoxObj> objs;
  long long total = 0;
  float max_abs = 0.0f;
  const aura_status_t s = voxel_objects(box_lo, box_hi, B, n_target, &objs, &total, &max_abs);
  if (s != AURA_OK) return s;
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    if (p1 < p0 || p0 < 0 || p1 > N || p1 - p0 > 0x7fffffff) return AURA_ERR_SHAPE;
    if ((b == 0 && p0 != 0) || (b == B - 1 && p1 != N)) return AURA_ERR_SHAPE;
    objs[(size_t)b].pt_begin = p0;
    objs[(size_t)b].n_pts = (int)(p1 - p0);
  }
  if (!out_offsets || (out_capacity > 0 && !out_xyz) || (N > 0 && !xyz)) return AURA_ERR_NULL;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < aura::voxel_workspace_bytes(total))
    return AURA_ERR_WORKSPACE;
  return hip_status(aura::launch_voxel_downsample(xyz, objs.data(), B, max_abs, N, out_xyz, out_count, out_capacity,
                                                  out_offsets, voxel_of_point, workspace,
                                                  static_cast<hipStream_t>(stream)));
}

aura_status_t aura_time_next_fusion(void* start_event, void* stop_event) {
  if ((start_event == nullptr) != (stop_event == nullptr)) return AURA_ERR_NULL;
  g_timing.start = static_cast<hipEvent_t>(start_event);
  g_timing.stop = static_cast<hipEvent_t>(stop_event);
  return AURA_OK;
}

aura_status_t aura_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (bytes == 0) return AURA_OK;
  if (!dst || !src) return AURA_ERR_NULL;
  if (bytes % 16 != 0) return AURA_ERR_SHAPE;
  if (!aligned(dst, 16) || !aligned(src, 16)) return AURA_ERR_ALIGN;
  return hip_status(aura::launch_calibration_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
}

aura_status_t aura_calibration_fill(void* dst, size_t bytes, uint32_t value, void* stream) {
  if (bytes == 0) return AURA_OK;
  if (!dst) return AURA_ERR_NULL;
  if (bytes % 16 != 0) return AURA_ERR_SHAPE;
  if (!aligned(dst, 16)) return AURA_ERR_ALIGN;
  return hip_status(aura::launch_calibration_fill(dst, bytes, value, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
