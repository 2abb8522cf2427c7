/*
 * libaura_fuse - multi-view semantic feature fusion onto a 3-D point / voxel set, per-point
 * material scoring and property integration, for AMD MI355X (gfx950).
 *
 * The calls follow the method of "Accelerating Physical Property Reasoning for Augmented
 * Visual Cognition" (AURA, arXiv 2511.03126):
 *   aura_project_visibility   Sec. 3.1 "Visibility Checking", Eq. 1
 *   aura_fuse_features        Sec. 3.1 "Feature Aggregation", Eq. 2 (+ L2 normalisation, implied
 *                             by the cosine similarity of Sec. 3.4.1)
 *   aura_material_scores      Sec. 3.4.1: similarity omega_k and the kernel regression of Eq. 4
 *   aura_voxel_downsample     Sec. 3.2.1: adaptive voxel size and voxel down-sampling of the point cloud
 *   aura_estimate_normals     Sec. 3.2.2: normals of the sampled points (input of the view importance score)
 *   aura_select_views         Sec. 3.2.2: view importance scores and the top-k views per point
 *   aura_fuse_selected        Sec. 3.2.3: Eq. 2 over the kept views only
 *   aura_patch_batch          Sec. 3.2.3: the multi-scale image patches of the kept views as one batch for the encoder
 *   aura_fuse_scores          aura_fuse_features and aura_material_scores in one (Eq. 2, then Sec. 3.4.1 / Eq. 4)
 *   aura_fuse_score_integrate Eq. 1-2, Sec. 3.4.1 / Eq. 4 and Sec. 3.4.2 in one pass that never writes the fused features
 *   aura_knn_densify          Sec. 3.4.1 Eq. 5: feature-space k-NN densification, then Eq. 4
 *   aura_property_integrate   Sec. 3.4.2: property times voxel volume, summed per object (mass)
 *   aura_thickness_integrate  Sec. 3.4.2: thickness-based integration (b_adap x b_adap x theta voxels, factor
 *                             lambda) and the centre of mass of Sec. 2.1 / 3.4
 *
 * General rules
 *   - Plain C ABI.  Every function returns an aura_status_t (0 = AURA_OK, negative = error);
 *     nothing throws, aborts or prints.
 *   - Pointers marked [device] are GPU global memory owned by the caller and must stay valid
 *     until the work enqueued on `stream` has finished.  Pointers marked [host] are ordinary
 *     host memory that is read before the call returns.  The library allocates and frees
 *     nothing and keeps no pointer after a call returns.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null stream).
 *     No call synchronises the stream or the device and no result is copied to the host.
 *   - Arrays are dense, row-major, innermost index last.  Results are a deterministic function
 *     of the inputs: the same call gives bitwise the same output.
 *   - Objects.  A call may cover B independent objects.  Object b owns points
 *     pt_offsets[b] .. pt_offsets[b+1]-1 of the concatenated point array and views
 *     view_offsets[b] .. view_offsets[b+1]-1 of the concatenated view arrays; a point is only
 *     ever tested against the views of its own object.  pt_offsets / view_offsets may both be
 *     NULL when B == 1 (one object: all points, all views).  All views of a call share
 *     H, W, Hf, Wf, D and the feature element type.
 *   - N == 0 is valid and does nothing.
 */
#ifndef AURA_FUSE_H
#define AURA_FUSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t aura_status_t;

enum {
  AURA_OK = 0,
  AURA_ERR_NULL = -1,        /* a required pointer is NULL                                   */
  AURA_ERR_SHAPE = -2,       /* a size is out of range or the offsets are inconsistent       */
  AURA_ERR_DTYPE = -3,       /* unknown element type                                         */
  AURA_ERR_ALIGN = -4,       /* a pointer or row pitch is not aligned as documented          */
  AURA_ERR_WORKSPACE = -5,   /* workspace missing or smaller than aura_workspace_bytes says  */
  AURA_ERR_HIP = -6,         /* a HIP call failed; see aura_last_hip_error()                 */
  AURA_ERR_UNSUPPORTED = -7  /* valid request this build has no kernel for                   */
};

/* Element type of the feature maps. */
enum { AURA_F32 = 0, AURA_BF16 = 1, AURA_F16 = 2 };

/* aura_params_t.flags */
enum {
  AURA_VIS_FRUSTUM_ONLY = 1u,  /* skip the depth comparison of Eq. 1: visible = in front of the
                                  camera and inside the image                                  */
  AURA_FUSE_MEAN_ONLY = 2u,    /* aura_fuse_features returns the plain mean of Eq. 2 without the
                                  L2 normalisation                                             */
  AURA_FUSE_GATHER = 4u,       /* aura_fuse_features uses the per-point gather kernel even where the
                                  matrix-core kernels apply (16-bit maps, D a multiple of 256).
                                  Meant for point sets that are not spatially sorted            */
  AURA_FUSE_TWO_KERNELS = 8u   /* the matrix-core fusion runs as two kernels (lists, then products) even where
                                  its one-kernel form applies, and aura_fuse_scores scores with a kernel of its
                                  own; same results bit for bit wherever every tile's cell list fits the
                                  one-kernel form's on-chip buffer (a longer list is fused there by the gather
                                  arithmetic, which can differ in the last bit)                 */,
  AURA_UNSEEN_PRIOR = 0u,      /* default.  A point that no view sees (Eq. 2 is 0 / 0 there: all-zero fused row, view
                                  count 0) has similarity 0 to every material, so Eq. 4 gives it the plain mean of y -
                                  the value before any observation.  It never enters an integral: aura_property_integrate
                                  and aura_thickness_integrate skip points whose count is 0                       */
  AURA_UNSEEN_ZERO = 16u       /* the scoring calls write 0 instead of that mean into the properties of a point whose
                                  similarities are all exactly zero (what an all-zero fused row gives): property fields
                                  in which "not observed" must not look like a material.  Scores and labels unchanged  */
};

/* Which call a workspace size is asked for. */
enum { AURA_CALL_MATERIAL_SCORES = 1, AURA_CALL_PROPERTY_INTEGRATE = 2, AURA_CALL_FUSE_FEATURES = 3,
       AURA_CALL_FUSE_SCORES = 4, AURA_CALL_KNN_DENSIFY = 5,
       AURA_CALL_THICKNESS_INTEGRATE = 6, AURA_CALL_FUSE_SCORE_INTEGRATE = 7 };

/* Problem sizes for aura_workspace_bytes; fields a call does not list are ignored. */
typedef struct aura_sizes_t {
  int64_t N;            /* points                                                              */
  int32_t B;            /* objects                                                             */
  int32_t n_views;      /* views over all objects                                              */
  int32_t Hf, Wf, D;    /* feature grid and channel count                                      */
  int32_t feat_dtype;   /* AURA_F32 | AURA_BF16 | AURA_F16                                     */
  int32_t K;            /* candidate materials                                                 */
  int32_t G;            /* voxels per axis of the integration grid, 0 = point-volume mode      */
  int32_t Ns;           /* source points of aura_knn_densify                                   */
  int32_t P;            /* property columns                                                    */
} aura_sizes_t;

/* One set of calibrated views (Sec. 3.1: poses, Depth_v and F_v for v in V). */
typedef struct aura_views_t {
  int32_t n_views;      /* total number of views over all objects, >= 1                       */
  int32_t H, W;         /* depth-map (= image) size in pixels                                  */
  int32_t Hf, Wf, D;    /* feature grid size and channel count                                 */
  int32_t feat_dtype;   /* AURA_F32 | AURA_BF16 | AURA_F16                                     */
  const float* cam;     /* [device] [n_views][16]: R (3x3 row-major), t (3), fx, fy, cx, cy.
                           Camera frame Xc = R x + t with +z forward, +x right, +y down;
                           pixel u = fx Xc.x / Xc.z + cx, v = fy Xc.y / Xc.z + cy, with pixel
                           (row r, column c) covering [c, c+1) x [r, r+1)                      */
  const float* depth;   /* [device] [n_views][H][W] depth along the camera z axis.  A texel that
                           is <= 0 or NaN is invalid (nothing is visible there); +inf means
                           nothing is in front.  May be NULL with AURA_VIS_FRUSTUM_ONLY        */
  const void* feat;     /* [device] [n_views][Hf][Wf][D] feature maps, channel last, 16-byte
                           aligned.  The grid covers the whole image: cell (r, c) is centred at
                           pixel coordinate ((c + 0.5) W / Wf, (r + 0.5) H / Hf).
                           Unused by aura_project_visibility                                   */
} aura_views_t;

typedef struct aura_params_t {
  float tau;            /* depth tolerance in scene units: visible iff proj_depth <= Depth + tau.
                           0 is Eq. 1 as printed                                               */
  float z_near;         /* points with camera-frame z <= z_near are invisible (e.g. 1e-6)      */
  float temperature;    /* T of Eq. 4, > 0; the paper uses 0.1                                  */
  float norm_eps;       /* L2 normalisation divides by max(norm, norm_eps) (e.g. 1e-12)        */
  uint32_t flags;       /* AURA_VIS_FRUSTUM_ONLY | AURA_FUSE_MEAN_ONLY | AURA_FUSE_GATHER | ...    */
} aura_params_t;

/* Library version as major * 10000 + minor * 100 + patch. */
int32_t aura_version(void);

/* Static, human-readable text for a status code. */
const char* aura_strerror(aura_status_t status);

/* The hipError_t of the last failed HIP call made by this thread (0 if none). */
int32_t aura_last_hip_error(void);

/*
 * Bytes of device scratch the given call needs (written to *bytes; may be 0).  The workspace
 * must be 256-byte aligned.  Only the fields listed matter:
 *   AURA_CALL_MATERIAL_SCORES     D, K
 *   AURA_CALL_PROPERTY_INTEGRATE  N, B, G
 *   AURA_CALL_FUSE_FEATURES       N, B, n_views, Hf, Wf, D, feat_dtype
 *   AURA_CALL_FUSE_SCORES         N, B, n_views, Hf, Wf, D, feat_dtype, K
 *   AURA_CALL_KNN_DENSIFY         D, Ns
 *   AURA_CALL_THICKNESS_INTEGRATE N, B
 *   AURA_CALL_FUSE_SCORE_INTEGRATE N, B, n_views, Hf, Wf, D, feat_dtype, K, P, G
 * Errors: AURA_ERR_NULL (sizes, bytes), AURA_ERR_SHAPE, AURA_ERR_DTYPE, AURA_ERR_UNSUPPORTED
 * (unknown call, or sizes beyond the limits of the call).
 */
aura_status_t aura_workspace_bytes(int32_t call, const aura_sizes_t* sizes, size_t* bytes);

/*
 * Where the status word of a fusion call lies inside its workspace.  The one-kernel form of the matrix-core fusion
 * (see aura_fuse_features) lets the waves that build a tile's cell lists wait for one another with a bounded number of
 * looks; should such a wait ever run out (it cannot, short of a defect in the library or the machine), the kernel
 * still ends, the results of the call are not to be trusted, and bit 0 of this 32-bit word is set.  Every call clears
 * the word when it starts.  The library never copies to the host: a caller who wants the guarantee reads the word
 * (workspace + *offset, device memory) after the stream has passed the call; zero means nothing to report.
 * The 32-bit word after it (workspace + *offset + 4) counts the tiles of 32 consecutive points whose list of touched
 * feature cells outgrew its storage and which were therefore fused point by point inside the kernel: correct, but many
 * times slower than either path at its best.  Spatially sorted points that are dense against the feature cells give
 * 0 or a handful; a count near N / 32 says that the 32 points of a tile lie too far apart for this path (points not
 * sorted, or far sparser than the cells): sort them (Morton order), or pass AURA_FUSE_GATHER.
 *   call  AURA_CALL_FUSE_FEATURES (also for aura_fuse_selected), AURA_CALL_FUSE_SCORES or AURA_CALL_FUSE_SCORE_INTEGRATE
 *   sizes as for aura_workspace_bytes     *present = 0: these sizes run kernels that have no such wait (no word)
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_DTYPE, AURA_ERR_UNSUPPORTED (another call).
 */
aura_status_t aura_fuse_status_offset(int32_t call, const aura_sizes_t* sizes, size_t* offset, int32_t* present);

/*
 * Sec. 3.1 "Visibility Checking", Eq. 1.  Projects every point into every view of its object
 * and evaluates the visibility mask
 *     M_vis(x_i, v) = [ z > z_near ] [ 0 <= u < W ] [ 0 <= v < H ] [ Depth_v valid ]
 *                     [ z <= Depth_v(floor(v), floor(u)) + tau ].
 * All of it is fp32 with one fixed operation order (three fused multiply-adds per camera-frame
 * coordinate starting from t, one division, one fused multiply-add for the pixel coordinate),
 * so the mask is reproducible bit for bit.
 *
 *   xyz    [device] [N][3] fp32 world coordinates
 *   pt_offsets [host] [B+1] int64, view_offsets [host] [B+1] int32 (or both NULL, B == 1)
 *   vis    [device] [N][vis_pitch] uint8: vis[i][j] = mask for the j-th view of i's object, 0 for
 *          j beyond the object's view count.  vis_pitch >= the largest per-object view count
 *   count  [device] [N] int32 = number of views that see the point (may be NULL)
 *   uvz    [device] [N][vis_pitch][3] fp32 (u, v, proj_depth), or NULL (debug output)
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_HIP.
 */
aura_status_t aura_project_visibility(const aura_views_t* views, const aura_params_t* params,
                                      const float* xyz, int64_t N,
                                      const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                      uint8_t* vis, int32_t vis_pitch, int32_t* count, float* uvz,
                                      void* stream);

/*
 * Sec. 3.1 "Feature Aggregation", Eq. 2.  For every point: bilinear samples of the feature maps
 * of the views that see it (the same mask as aura_project_visibility, recomputed), averaged,
 * then divided by max(L2 norm, norm_eps) unless AURA_FUSE_MEAN_ONLY.  Sampling: grid coordinate
 * g = u / (W / Wf) - 0.5 (same in v), clamped to [0, Wf - 1]; the four cells around g are blended
 * with weights from the fractional part.  Half-precision elements are widened exactly; all
 * arithmetic and the output are fp32.  A point no view sees gets an all-zero row.
 *
 *   fused  [device] [N][D] fp32, 16-byte aligned
 *   count  [device] [N] int32 or NULL
 *   workspace [device] aura_workspace_bytes(AURA_CALL_FUSE_FEATURES, ...) bytes, 256-byte aligned,
 *          or NULL.  With a workspace, 16-bit maps whose D is a multiple of 256 (up to 1536, except
 *          1280; maps below 4 GiB) run on the matrix cores: the
 *          points are taken 32 at a time and should arrive spatially sorted (e.g. Morton order),
 *          and the maps must be finite everywhere.  Without one, or for other shapes, or with
 *          AURA_FUSE_GATHER, a per-point gather kernel is used.  Both give the same result up to
 *          fp32 rounding.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_DTYPE, AURA_ERR_ALIGN (feat or fused not
 * 16-byte aligned), AURA_ERR_WORKSPACE (given but misaligned or too small), AURA_ERR_HIP.
 */
aura_status_t aura_fuse_features(const aura_views_t* views, const aura_params_t* params,
                                 const float* xyz, int64_t N,
                                 const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                 float* fused, int32_t* count,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.4.1.  scores[i][k] = <fused_i, temb_k> (the cosine similarity omega_k when both are
 * unit vectors; temb is used as given), and, when y is given, Eq. 4:
 *     prop[i][p] = sum_k exp(scores[i][k] / T) y[k][p] / sum_k exp(scores[i][k] / T),
 * evaluated with the row maximum subtracted.  label[i] = argmax_k scores[i][k], the lowest k
 * on exact ties.  An all-zero fused row therefore gives the plain mean of y and label 0.
 *
 *   fused  [device] [N][D] fp32          temb  [device] [K][D] of temb_dtype (AURA_F32, AURA_BF16 or AURA_F16;
 *          16-bit embeddings are widened exactly to fp32 first, into the workspace)
 *   y      [device] [K][P] fp32 or NULL  scores [device] [N][K] fp32
 *   prop   [device] [N][P] fp32 or NULL (needs y)   label [device] [N] int32 or NULL
 *   workspace [device] aura_workspace_bytes(AURA_CALL_MATERIAL_SCORES, ...) bytes, 256-byte aligned
 * The products run on the matrix cores with each fp32 operand split into two bf16 terms (three
 * partial products), accumulated in fp32: absolute error of a score is below 1e-5 for unit vectors.
 * Limits: 1 <= K <= 128, 1 <= P <= 8.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_DTYPE, AURA_ERR_WORKSPACE, AURA_ERR_UNSUPPORTED
 * (K or P beyond the limits), AURA_ERR_HIP.
 */
aura_status_t aura_material_scores(const float* fused, int64_t N, int32_t D,
                                   const void* temb, int32_t temb_dtype, int32_t K,
                                   const float* y, int32_t P, const aura_params_t* params,
                                   float* scores, float* prop, int32_t* label,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * aura_material_scores for callers that cannot allocate device memory or hand over a workspace: code that runs under
 * stream capture, serving loops with a fixed memory plan, harnesses that forbid allocation.  Same arguments (without
 * the workspace), same kernels, same results bit for bit.  The scratch of the call (the text embeddings split into
 * two 16-bit terms, ceil(D / 32) * ceil(K / 32) * 4096 bytes, three tiles of materials counted as four, plus 4 K D bytes
 * for the fp32 copy of 16-bit embeddings) lives in a
 * fixed array of AURA_STATIC_SCRATCH_BYTES inside the library's device image: every GPU the library is used on holds
 * that array until the process ends, and shapes that need more are refused.  The call allocates and frees nothing.
 * It works on the GPU that is current when it is called, and `stream` must belong to that GPU.  All calls on one GPU
 * share the array: two calls whose work overlaps in time on the same GPU (different streams, or different host
 * threads) race on it and give undefined scores; calls on one stream are ordered and safe.  Each call rewrites the
 * part of the array it reads, so nothing of an earlier call is seen.
 * Errors: those of aura_material_scores except AURA_ERR_WORKSPACE; AURA_ERR_UNSUPPORTED also when D and K need more
 * scratch than the array holds (e.g. D = 4096 with K = 128: 4 MiB); AURA_ERR_HIP when the array cannot be located.
 */
#define AURA_STATIC_SCRATCH_BYTES (2u << 20)
aura_status_t aura_material_scores_static(const float* fused, int64_t N, int32_t D,
                                          const void* temb, int32_t temb_dtype, int32_t K,
                                          const float* y, int32_t P, const aura_params_t* params,
                                          float* scores, float* prop, int32_t* label, void* stream);

/*
 * Sec. 3.1 Eq. 1 and 2 followed by Sec. 3.4.1 / Eq. 4 in one call: everything aura_fuse_features writes
 * (fused, count), optionally the mask of aura_project_visibility, and everything aura_material_scores writes (scores, prop, label) for the same
 * points, with the arguments and rules of those two calls.
 *
 * The similarity omega_k = <f, t_k> is linear in f, and the fused feature is a weighted sum of
 * feature cells.  Where the fusion runs on the matrix cores (see aura_fuse_features) and the call has
 * no more feature cells (n_views * Hf * Wf) than points, the library therefore first computes the
 * similarity of every feature cell to every material and then applies the fusion weights of each
 * point to those K numbers instead of to the D channels; the fused rows are written but never read
 * back.  This is the same sum in another order: scores agree with
 * aura_material_scores(aura_fuse_features(...)) up to fp32 rounding (the per-cell similarities and the
 * weights are carried as two 16-bit terms each, about 16 mantissa bits).  In every other case the
 * call is exactly the two calls in sequence.
 *
 *   fused  [device] [N][D] fp32, 16-byte aligned (required)    count [device] [N] int32 or NULL
 *   vis    [device] [N][vis_pitch] uint8 or NULL: the mask of Eq. 1 exactly as aura_project_visibility writes it
 *          (the fusion evaluates it anyway), vis_pitch >= the largest per-object view count
 *   temb   [device] [K][D] of temb_dtype (AURA_F32, AURA_BF16 or AURA_F16)  y     [device] [K][P] fp32 or NULL
 *   scores [device] [N][K] fp32   prop [device] [N][P] fp32 or NULL (needs y)   label [device] [N] or NULL
 *   workspace [device] aura_workspace_bytes(AURA_CALL_FUSE_SCORES, ...) bytes, 256-byte aligned (required)
 * Limits: 1 <= K <= 128, 1 <= P <= 8.
 * Errors: those of aura_fuse_features and aura_material_scores.
 */
aura_status_t aura_fuse_scores(const aura_views_t* views, const aura_params_t* params,
                               const float* xyz, int64_t N,
                               const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                               const void* temb, int32_t temb_dtype, int32_t K, const float* y, int32_t P,
                               float* fused, int32_t* count, uint8_t* vis, int32_t vis_pitch,
                               float* scores, float* prop, int32_t* label,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.1 Eq. 1-2, then Sec. 3.4.1 / Eq. 4, then Sec. 3.4.2 (the voxel sum of property times volume), in one pass: what
 * aura_fuse_scores followed by aura_property_integrate (column p_index of the properties, the view counts of the
 * fusion as `count`) computes, for callers that want scores, property fields and the integrated property but not the
 * fused features themselves.  Sec. 3.4.1 and 3.4.2 consume only omega, rho and the mass; the fused feature of Eq. 2 is
 * an intermediate, and here its [N][D] array is never written to memory:
 *   - where the fusion runs on the matrix cores (see aura_fuse_features) and the call has at most four times as many
 *     feature cells as points, the scores come from per-cell similarities as in aura_fuse_scores, the fusion kernels
 *     keep each tile's rows in registers only as long as the L2 norm needs them;
 *   - otherwise the rows of 32768 points at a time pass through a buffer in the workspace between the gather kernel and
 *     the scoring kernel.
 * Results equal those of the two calls up to fp32 rounding (bit for bit where aura_fuse_scores takes the same kernels).
 * Arguments as in aura_fuse_scores and aura_property_integrate, except:
 *   y      [device] [K][P] fp32, required (P >= 1)
 *   count  [device] [N] int32 or NULL     vis [device] [N][vis_pitch] uint8 or NULL
 *   scores [device] [N][K] fp32 (required)   prop [device] [N][P] fp32 or NULL   label [device] [N] int32 or NULL
 *   mass   [device] [B] fp32 (required)   n_used [device] [B] int64 or NULL
 *   workspace [device] aura_workspace_bytes(AURA_CALL_FUSE_SCORE_INTEGRATE, ...) bytes, 256-byte aligned (required)
 * A point no view sees has scores 0 and the mean of y as its property (0 with AURA_UNSEEN_ZERO), and does not enter
 * the mass.
 * Errors: those of aura_fuse_scores and aura_property_integrate.
 */
aura_status_t aura_fuse_score_integrate(const aura_views_t* views, const aura_params_t* params,
                                        const float* xyz, int64_t N,
                                        const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                        const void* temb, int32_t temb_dtype, int32_t K, const float* y, int32_t P,
                                        int32_t p_index, const float* vol, float vol_uniform,
                                        const float* grid_lo, const float* grid_h, int32_t G,
                                        int32_t* count, uint8_t* vis, int32_t vis_pitch,
                                        float* scores, float* prop, int32_t* label,
                                        float* mass, int64_t* n_used,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.4.1 Eq. 5, densification.  Ns sparse source points carry material vectors ws[j] (the K numbers
 * that Eq. 4 consumes, e.g. the scores of aura_material_scores at those points); every dense query point
 * gets the similarity-weighted mean of the vectors of its k nearest sources in feature space:
 *     phi_j = cosine similarity of fq[i] and fs[j]  (0 when either vector is zero),
 *     N_k(i) = the k sources with the largest phi (of equal values the lower index first; k is cut to Ns),
 *     wq[i][m] = sum_{j in N_k(i)} phi_j ws[j][m] / sum_{j in N_k(i)} phi_j.
 * Eq. 5 is taken as printed: the weights are the similarities themselves, negative ones included; when the
 * sum of the weights is below 1e-12 in magnitude the vector of the nearest source is returned.  Then Eq. 4 on
 * wq[i] when y is given: prop[i][p] = sum_m softmax_m(wq[i] / T) y[m][p]; label[i] = argmax_m wq[i][m].
 * The paper does not print its k: it is an argument.
 *
 *   fq  [device] [Nq][D] fp32 features of the queries (e.g. the rows of aura_fuse_features)
 *   fs  [device] [Ns][D] fp32 features of the source points       ws [device] [Ns][K] fp32
 *   y   [device] [K][P] fp32 or NULL      wq [device] [Nq][K] fp32
 *   prop [device] [Nq][P] fp32 or NULL (needs y)   label [device] [Nq] int32 or NULL
 *   nn_idx [device] [Nq][k] int32 or NULL: the neighbours in selection order (-1 beyond Ns)
 *   workspace [device] aura_workspace_bytes(AURA_CALL_KNN_DENSIFY, ...) bytes, 256-byte aligned
 * The similarities run on the matrix cores with each fp32 operand split into two bf16 terms (error of a
 * similarity near 1e-6), so which of two sources closer than that is "nearer" may differ from an exact
 * evaluation.  A NaN among a query's features makes its similarities unordered: its outputs are then
 * unspecified (its nn_idx entries still name sources of the set), the other queries are not affected; a source
 * whose features hold a NaN is never selected.
 * Limits: 1 <= Ns <= 256, 1 <= k <= 16, 1 <= K <= 128, 1 <= P <= 8.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_WORKSPACE, AURA_ERR_UNSUPPORTED, AURA_ERR_HIP.
 */
aura_status_t aura_knn_densify(const float* fq, int64_t Nq, int32_t D, const float* fs, int32_t Ns,
                               const float* ws, int32_t K, int32_t k, const float* y, int32_t P,
                               const aura_params_t* params, float* wq, float* prop, int32_t* label,
                               int32_t* nn_idx, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.4.2, integration of a property over voxels.  Each point is the centre of a voxel; the
 * integrated property of object b is the sum of property times voxel volume.  A point is used
 * when count is NULL or count[i] > 0.
 *   G == 0, point-volume mode:  mass[b] = sum_i prop[i][p_index] * vol_i,  vol_i = vol[i] if vol is
 *           given, else vol_uniform.
 *   G  > 0, grid mode: object b has a cube of G^3 voxels of side grid_h[b] whose lower corner is
 *           grid_lo[b].  A point falls in voxel clamp(floor((x - lo) * (1 / h)), 0, G - 1) per axis
 *           (fp32).  mass[b] = h^3 * sum over occupied voxels of the mean property of the used
 *           points inside.
 * Products are fp32, sums are exact (fixed point) or fp64 in a fixed order.
 *
 *   prop   [device] [N][P] fp32          count [device] [N] int32 or NULL
 *   vol    [device] [N] fp32 or NULL     pt_offsets [host] [B+1] int64 or NULL (B == 1)
 *   xyz    [device] [N][3] fp32 (grid mode)   grid_lo [host] [B][3] fp32, grid_h [host] [B] fp32
 *   mass   [device] [B] fp32             n_used [device] [B] int64 or NULL
 *   workspace [device] aura_workspace_bytes(AURA_CALL_PROPERTY_INTEGRATE, ...) bytes
 * Limits: B <= 4096; G <= 512 and B * G^3 < 2^31 in grid mode.  prop must be finite.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_WORKSPACE, AURA_ERR_UNSUPPORTED, AURA_ERR_HIP.
 */
aura_status_t aura_property_integrate(const float* prop, int64_t N, int32_t P, int32_t p_index,
                                      const int32_t* count, const float* vol, float vol_uniform,
                                      const int64_t* pt_offsets, int32_t B,
                                      const float* xyz, const float* grid_lo, const float* grid_h, int32_t G,
                                      float* mass, int64_t* n_used,
                                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.2.1 "Adaptive Sampling".  The voxel size follows the object instead of being fixed,
 *     s_voxel = cbrt(V_bound / N_target),
 * V_bound the volume of the boundary box of the point cloud and N_target the wanted number of points (the paper takes
 * about 150); the box is cut into cubes of side s_voxel and every occupied cube is replaced by the mean position of
 * its points (standard voxel down-sampling).
 * Arithmetic that decides an integer is fp32: extents e = hi - lo; s_voxel = (float)cbrt((double)e_x e_y e_z /
 * N_target); a box without volume takes e_max / cbrt(N_target), a box of one point 1; cubes per axis
 * floor(e / s_voxel) + 1; a point's cube per axis clamp(floor((x - lo) / s_voxel), 0, cubes - 1).  Sums are exact
 * (64-bit fixed point), so the result does not depend on the order of the points.
 *
 * aura_voxel_grid (host only, no GPU work): s_voxel and the cubes per axis (dims[3]) of one box.
 * aura_voxel_workspace_bytes: workspace of aura_voxel_downsample for these boxes.
 * aura_voxel_downsample:
 *   xyz [device] [N][3] fp32          pt_offsets [host] [B+1] int64 or NULL (B == 1)
 *   box_lo, box_hi [host] [B][3] fp32: the boundary box of every object (hi >= lo).  Points outside it fall into its
 *           border cubes; they may lie up to one box extent outside.
 *   out_xyz [device] [out_capacity][3] fp32: the sampled points, object after object, inside an object in the order
 *           of the cube index (z * ny + y) * nx + x          out_count [device] [out_capacity] int32 or NULL: points per cube
 *   out_offsets [device] [B+1] int32: range of every object in the list; out_offsets[B] is the number of occupied
 *           cubes even when it exceeds out_capacity (the cubes beyond it are not written)
 *   voxel_of_point [device] [N] int32 or NULL: list position of the point's cube
 *   workspace [device] aura_voxel_workspace_bytes(...) bytes, 256-byte aligned
 * Limits: B <= 64; the grids of a call hold at most 2^24 cubes in all (every object rounded up to 2048).
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_WORKSPACE, AURA_ERR_UNSUPPORTED, AURA_ERR_HIP.
 */
aura_status_t aura_voxel_grid(const float* box_lo, const float* box_hi, int32_t n_target, float* s_voxel, int32_t* dims);
aura_status_t aura_voxel_workspace_bytes(const float* box_lo, const float* box_hi, int32_t B, int32_t n_target,
                                         size_t* bytes);
aura_status_t aura_voxel_downsample(const float* xyz, int64_t N, const int64_t* pt_offsets, int32_t B,
                                    const float* box_lo, const float* box_hi, int32_t n_target, float* out_xyz,
                                    int32_t* out_count, int64_t out_capacity, int32_t* out_offsets,
                                    int32_t* voxel_of_point, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.2.2, the normals of the sampled points that the view importance score needs.  For every query point q of
 * object b: the k points of the object's cloud nearest to q; the normal is the unit eigenvector of the smallest
 * eigenvalue of their covariance (the plane through them), with the sign that points away from centre[b]
 * (the outward orientation the section asks for; when it is at right angles to q - centre the sign is arbitrary).  The paper names no
 * neighbourhood size: k is an argument.
 * Which points are nearest is decided on the fp32 distance d = (dx dx + dy dy) + dz dz, dx = p_x - q_x, every
 * operation rounded to fp32; of equal distances the lower index first.  Sums, covariance and eigenvectors are fp64.
 * An object with fewer than k points uses all of them; without points the normal is 0.
 *
 *   xyz [device] [N][3] fp32: the clouds          pt_offsets [host] [B+1] int64 or NULL (B == 1)
 *   queries [device] [M][3] fp32                   q_offsets  [host] [B+1] int64 or NULL (with pt_offsets)
 *   centre [host] [B][3] fp32: a point inside every object (e.g. the centroid of its cloud)
 *   normals [device] [M][3] fp32                   evals [device] [M][3] fp32 or NULL: eigenvalues, ascending
 * Limits: B <= 4096.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_UNSUPPORTED, AURA_ERR_HIP.
 */
aura_status_t aura_estimate_normals(const float* xyz, int64_t N, const int64_t* pt_offsets, const float* queries, int64_t M,
                                    const int64_t* q_offsets, int32_t B, const float* centre, int32_t k, float* normals,
                                    float* evals, void* stream);

/*
 * Sec. 3.2.2 "View Importance-based Filtering".  For every visible pair (Eq. 1, as aura_project_visibility):
 *     S_dist = 1 / (1 + z)             z: depth of the point in the camera frame
 *     S_angle = max(0, v . (-n))       v: unit vector from the camera centre to the point, n: unit normal of the point
 *     S_total = S_dist * S_angle
 * and the k visible views with the largest S_total are kept for the point (of equal scores the lower view index
 * first; a visible view that sees the back of the surface has score 0 and is kept only when fewer than k views score
 * higher).  The paper keeps k = 3.  Scores are fp32.
 *
 *   xyz, normals [device] [N][3] fp32 (normals of unit length, oriented outward)
 *   pt_offsets, view_offsets [host] as in aura_project_visibility
 *   sel_view  [device] [N][k] int32: kept views in rank order, as indices within the object; -1 beyond the visible ones
 *   sel_score [device] [N][k] fp32 or NULL: their S_total (0 beyond)
 *   sel_mask  [device] [N][mask_pitch] uint8 or NULL: 1 for kept pairs, 0 elsewhere; mask_pitch >= views per object
 *   n_sel     [device] [N] int32 or NULL: number of kept views, min(k, visible views)
 * Limits: 1 <= k <= 8.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_UNSUPPORTED, AURA_ERR_HIP.
 */
aura_status_t aura_select_views(const aura_views_t* views, const aura_params_t* params, const float* xyz,
                                const float* normals, int64_t N, const int64_t* pt_offsets,
                                const int32_t* view_offsets, int32_t B, int32_t k, int32_t* sel_view, float* sel_score,
                                uint8_t* sel_mask, int32_t mask_pitch, int32_t* n_sel, void* stream);

/*
 * Sec. 3.2.3: the features of the kept views are fused by averaging.  aura_fuse_features with the weight of a pair
 * taken from sel_mask (e.g. the output of aura_select_views) instead of Eq. 1: fused[i] = mean over
 * {v : sel_mask[i][v] != 0} of F_v(pi(x_i, v)), then L2 normalisation as in aura_fuse_features.  The depth maps are
 * not read (views->depth may be NULL); a kept pair that projects behind the camera or outside the image is ignored.
 * count [N] (or NULL) receives the number of views that entered the mean.  Everything else, the workspace
 * (AURA_CALL_FUSE_FEATURES) included, as for aura_fuse_features.
 *   sel_mask [device] [N][mask_pitch] uint8, mask_pitch >= views per object
 */
aura_status_t aura_fuse_selected(const aura_views_t* views, const aura_params_t* params, const float* xyz, int64_t N,
                                 const int64_t* pt_offsets, const int32_t* view_offsets, int32_t B,
                                 const uint8_t* sel_mask, int32_t mask_pitch, float* fused, int32_t* count,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.2.3 "Multi-scale Feature Fusion": the patches P_v^(l)(s).  For every source point s, each of its kept views
 * (sel_view, as written by aura_select_views: index within the object, -1 = none) and each scale l, the l x l pixel
 * square of the view's image centred at the projection pi(s, v) = (u, v) is resampled to R x R and written
 * channel-first into one batch for the image encoder (the paper uses three scales of 20, 40 and 60 pixels; the
 * encoder is not part of this library).  The image is read as a continuous field: bilinear between pixel centres at
 * integer + 0.5, the border pixel repeated outside the image; output pixel (i, j) samples it at
 *     x = u - l/2 + (j + 0.5) l / R,    y = v - l/2 + (i + 0.5) l / R
 * and stores (value / 255 - mean[c]) * inv_std[c].  A missing view gives a patch of zeros and valid = 0.
 *
 *   cam    [device] [n_views][16] fp32 as in aura_views_t           images [device] [n_views][H][W][3] uint8
 *   xyz    [device] [M][3] fp32             pt_offsets, view_offsets [host] as in aura_project_visibility
 *   sel_view [device] [M][k] int32          scales [host] [L] fp32 (> 0)
 *   mean, inv_std [host] [3] fp32 or NULL (0 and 1)
 *   out    [device] [M][k][L][3][R][R] of out_dtype (AURA_F32 or AURA_F16)       valid [device] [M][k] uint8 or NULL
 * Limits: L <= 8; M_b * k * L * ceil(R / 32) < 2^31 per object.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_DTYPE, AURA_ERR_ALIGN, AURA_ERR_UNSUPPORTED, AURA_ERR_HIP.
 */
aura_status_t aura_patch_batch(const float* cam, int32_t n_views, int32_t H, int32_t W, const uint8_t* images,
                               const float* xyz, int64_t M, const int64_t* pt_offsets, const int32_t* view_offsets,
                               int32_t B, const int32_t* sel_view, int32_t k, const float* scales, int32_t L, int32_t R,
                               const float* mean, const float* inv_std, void* out, int32_t out_dtype, uint8_t* valid,
                               void* stream);

/*
 * Sec. 3.4.2, thickness-based integration.  Every point s of object b is the centre of a voxel
 * b_adap x b_adap x theta_k, where b_adap^2 = A_bar = (L * scale_factor)^2 / N_b is the area one point stands
 * for (N_b: all points of the object):
 *     zeta[s]  = sum_k softmax_k(scores[s] / T)_k * y[k][p_index] * theta[k] * b_adap^2 * lambda
 *     total[b] = sum of zeta over the object's used points (count NULL or count[i] > 0): the mass when
 *                column p_index of y holds densities
 *     com[b]   = sum zeta[s] xyz[s] / total[b], the centre of mass (Sec. 2.1 names it among the integral
 *                estimates; zero when total[b] is 0)
 * L is box_len[b] when box_len is given, else the longest side of the axis-aligned bounding box of all the
 * object's points (the paper asks for a length that characterises the bounding box without choosing one).
 * T = params->temperature; the paper takes T = 0.1 and lambda = 0.6.  fp32 per point, fp64 sums in a fixed order.
 *
 *   scores [device] [N][K] fp32       y [device] [K][P] fp32       theta [device] [K] fp32
 *   xyz    [device] [N][3] fp32       count [device] [N] int32 or NULL
 *   pt_offsets [host] [B+1] int64 or NULL (B == 1)     box_len [host] [B] fp32 (>= 0) or NULL
 *   zeta   [device] [N] fp32 or NULL (0 for unused points)         total [device] [B] fp32
 *   com    [device] [B][3] fp32 or NULL   b_adap [device] [B] fp32 or NULL   n_used [device] [B] int64 or NULL
 *   workspace [device] aura_workspace_bytes(AURA_CALL_THICKNESS_INTEGRATE, ...) bytes, 256-byte aligned
 * Limits: K <= 128, B <= 4096.  scores must be finite.
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE, AURA_ERR_WORKSPACE, AURA_ERR_UNSUPPORTED, AURA_ERR_HIP.
 */
aura_status_t aura_thickness_integrate(const float* scores, int64_t N, int32_t K, const float* y, int32_t P,
                                       int32_t p_index, const float* theta, const float* xyz, const int32_t* count,
                                       const int64_t* pt_offsets, int32_t B, const float* box_len,
                                       const aura_params_t* params, float lambda, float scale_factor,
                                       float* zeta, float* total, float* com, float* b_adap, int64_t* n_used,
                                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Timing aid (not part of the method).  The next call of aura_fuse_features, aura_fuse_selected, aura_fuse_scores or
 * aura_fuse_score_integrate made by this host thread records start_event on its stream right before, and stop_event
 * right after, the launch of its fusion kernel (the kernel that evaluates Eq. 1-2 and writes the fused rows; both
 * kernels where the matrix-core fusion runs as two; of a call with more than 64 objects the first launch).  The time
 * between the two events is the kernel's duration plus what the two stream markers cost (some microseconds).  One shot:
 * the request is consumed by that launch.  Both NULL withdraws a pending request.  The benchmark uses it to time the
 * dominant kernel inside a call that launches several.
 *   start_event, stop_event  hipEvent_t created by the caller with timing enabled
 * Errors: AURA_ERR_NULL (exactly one of the two is NULL).
 */
aura_status_t aura_time_next_fusion(void* start_event, void* stop_event);

/*
 * Bandwidth calibration (not part of the method).  A plain copy of `bytes` bytes from src to dst,
 * and a plain fill of dst with a 32-bit pattern, each by one grid-stride kernel of 16-byte
 * accesses with streaming stores.  The benchmark times them to state what the memory system
 * delivers to the simplest kernel, and profiler byte counters are scaled by their reading for
 * these known sizes.
 *   dst, src [device] 16-byte aligned, not overlapping; bytes a multiple of 16 (0 does nothing)
 * Errors: AURA_ERR_NULL, AURA_ERR_SHAPE (bytes not a multiple of 16), AURA_ERR_ALIGN, AURA_ERR_HIP.
 */
aura_status_t aura_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);
aura_status_t aura_calibration_fill(void* dst, size_t bytes, uint32_t value, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AURA_FUSE_H */
