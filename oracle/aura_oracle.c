/*
 * CPU oracle for multi-view feature fusion, material scoring and property
 * integration (AURA, arXiv 2511.03126).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, per-point implementation of
 * the definitions in the paper, used to check the GPU library.  It shares no
 * code, header, table or helper with the GPU library and must never be called
 * from a product path.
 *
 * What each function follows:
 *   projection pi(x_i, v), proj_depth      Sec. 3.1 "Visibility Checking" (pinhole model;
 *                                          depth = z in the camera frame, Sec. 3.2.2)
 *   visibility mask M_vis                  Sec. 3.1 Eq. 1
 *   feature aggregation                    Sec. 3.1 Eq. 2 (bilinear sampling of F_v)
 *   similarity omega_k                     Sec. 3.4.1 (cosine similarity to text embedding k)
 *   kernel regression rho(s)               Sec. 3.4.1 Eq. 4, T from Sec. 4 "Parameters"
 *   integration to mass                    Sec. 3.4.2 (each query point is the centre of a
 *                                          voxel; property times voxel volume, summed)
 *   densification omega(q)                 Sec. 3.4.1 Eq. 5 (k nearest source points by cosine
 *                                          similarity of the fused features, similarity-weighted
 *                                          mean of their material vectors, then Eq. 4)
 *   adaptive sampling                      Sec. 3.2.1 (voxel size from the boundary box volume and N_target, voxel
 *                                          down-sampling to the mean position per occupied voxel)
 *   view importance-based filtering        Sec. 3.2.2 (S_dist, S_angle, S_total, top-k views per point) and the
 *                                          mean over the kept views of Sec. 3.2.3
 *   multi-scale patches                    Sec. 3.2.3 (squares of several sizes around the projection in each kept view,
 *                                          resampled into one batch for the encoder; the encoder itself is not here)
 *   thickness-based integration            Sec. 3.4.2 (voxel b_adap x b_adap x theta per point, correction
 *                                          factor lambda) and the centre of mass it gives
 *
 * Precision.  All sums, weights and outputs are double.  The few quantities that
 * DECIDE an integer (which depth texel is read, whether a point passes the depth
 * test, which four feature cells are blended, which grid voxel a point falls in)
 * are evaluated in fp32 with one fixed operation order, written out below with
 * fmaf(), so that an fp32 implementation can take the same decisions.  The same
 * quantities are also evaluated in double and the disagreements are reported as
 * diagnostics.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math).
 * The OpenMP pragma only distributes independent points over threads; every
 * point is still computed start to finish by the plain loop nest.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };
enum { ORC_FLAG_FRUSTUM_ONLY = 1, ORC_FLAG_MEAN_ONLY = 2 };
enum { ORC_DIAG_NEAR_THRESHOLD = 1, ORC_DIAG_NEAR_PIXEL_EDGE = 2, ORC_DIAG_F64_DIFFERS = 4 };

/* ---------------------------------------------------------------- element widening */

static float bits_to_float(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }

/* IEEE binary16 -> binary32, exact. */
static float half_to_float(uint16_t h) {
  uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  uint32_t exp = (h >> 10) & 0x1fu;
  uint32_t man = h & 0x3ffu;
  if (exp == 0) {
    if (man == 0) return bits_to_float(sign);
    /* subnormal: value = man * 2^-24 */
    float v = (float)man * 5.9604644775390625e-8f;
    return sign ? -v : v;
  }
  if (exp == 31) return bits_to_float(sign | 0x7f800000u | (man << 13));
  return bits_to_float(sign | ((exp + 112u) << 23) | (man << 13));
}

/* One stored feature element as a double (bf16 = upper half of a binary32). */
static double feat_at(const void* feat, int dtype, int64_t idx) {
  if (dtype == ORC_F32) return (double)((const float*)feat)[idx];
  if (dtype == ORC_BF16) return (double)bits_to_float((uint32_t)((const uint16_t*)feat)[idx] << 16);
  return (double)half_to_float(((const uint16_t*)feat)[idx]);
}

/* ---------------------------------------------------------------- a1: projection
 * cam = { R (row-major 3x3), t (3), fx, fy, cx, cy }; camera frame Xc = R x + t,
 * +z forward; u = fx*Xc.x/Xc.z + cx, v = fy*Xc.y/Xc.z + cy; proj_depth = Xc.z.   */

static void project_f32(const float* cam, const float* p, float* u, float* v, float* z) {
  float xc = fmaf(cam[2], p[2], fmaf(cam[1], p[1], fmaf(cam[0], p[0], cam[9])));
  float yc = fmaf(cam[5], p[2], fmaf(cam[4], p[1], fmaf(cam[3], p[0], cam[10])));
  float zc = fmaf(cam[8], p[2], fmaf(cam[7], p[1], fmaf(cam[6], p[0], cam[11])));
  float qx = xc / zc;
  float qy = yc / zc;
  *u = fmaf(cam[12], qx, cam[14]);
  *v = fmaf(cam[13], qy, cam[15]);
  *z = zc;
}

static void project_f64(const float* cam, const float* p, double* u, double* v, double* z) {
  double x = p[0], y = p[1], w = p[2];
  double xc = (double)cam[0] * x + (double)cam[1] * y + (double)cam[2] * w + (double)cam[9];
  double yc = (double)cam[3] * x + (double)cam[4] * y + (double)cam[5] * w + (double)cam[10];
  double zc = (double)cam[6] * x + (double)cam[7] * y + (double)cam[8] * w + (double)cam[11];
  *u = (double)cam[12] * (xc / zc) + (double)cam[14];
  *v = (double)cam[13] * (yc / zc) + (double)cam[15];
  *z = zc;
}

/* ---------------------------------------------------------------- a2: Eq. 1
 * Pixel (row r, col c) covers [c,c+1) x [r,r+1).  A point is visible when it is in
 * front of the camera, lands inside the image, the depth texel is valid (> 0; NaN
 * fails) and proj_depth <= Depth + tau.  tau = 0 is Eq. 1 as printed.             */

static int visible_f32(const float* depth_v, int H, int W, float tau, float z_near, int frustum_only,
                       float u, float v, float z) {
  int inside = (z > z_near) && (u >= 0.0f) && (u < (float)W) && (v >= 0.0f) && (v < (float)H);
  if (!inside) return 0;
  if (frustum_only) return 1;
  int px = (int)floorf(u), py = (int)floorf(v);
  float d = depth_v[(int64_t)py * W + px];
  if (!(d > 0.0f)) return 0;
  float lim = d + tau;
  return z <= lim;
}

static int visible_f64(const float* depth_v, int H, int W, float tau, float z_near, int frustum_only,
                       double u, double v, double z) {
  int inside = (z > (double)z_near) && (u >= 0.0) && (u < (double)W) && (v >= 0.0) && (v < (double)H);
  if (!inside) return 0;
  if (frustum_only) return 1;
  int px = (int)floor(u), py = (int)floor(v);
  double d = (double)depth_v[(int64_t)py * W + px];
  if (!(d > 0.0)) return 0;
  return z <= d + (double)tau;
}

static unsigned diag_flags(const float* cam, const float* depth_v, int H, int W, float tau, float z_near,
                           int frustum_only, const float* p, float u, float v, float z, int vis32) {
  unsigned f = 0;
  double ud, vd, zd;
  project_f64(cam, p, &ud, &vd, &zd);
  if (visible_f64(depth_v, H, W, tau, z_near, frustum_only, ud, vd, zd) != vis32) f |= ORC_DIAG_F64_DIFFERS;
  int inside = (z > z_near) && (u >= 0.0f) && (u < (float)W) && (v >= 0.0f) && (v < (float)H);
  if (fabs(ud - nearbyint(ud)) <= 1e-4 || fabs(vd - nearbyint(vd)) <= 1e-4) f |= ORC_DIAG_NEAR_PIXEL_EDGE;
  if (inside && !frustum_only) {
    double d = (double)depth_v[(int64_t)((int)floorf(v)) * W + (int)floorf(u)];
    if (d > 0.0 && isfinite(d)) {
      double scale = fabs(d) > 1.0 ? fabs(d) : 1.0;
      if (fabs(zd - (d + (double)tau)) <= 1e-5 * scale) f |= ORC_DIAG_NEAR_THRESHOLD;
    }
  }
  return f;
}

/* ---------------------------------------------------------------- a3: bilinear sample
 * The Hf x Wf grid covers the H x W image; cell k is centred at image coordinate
 * (k + 0.5) * pitch, pitch = W / Wf.  Grid coordinate g = u / pitch - 0.5, clamped to
 * [0, Wf-1] (replicated border).  g is taken in fp32 (pitch one fp32 division, then
 * one division and one subtraction), so an integer pitch puts cell centres exactly on
 * integers; the cell indices are floor(g) and the blend weights its exact fractional
 * part, carried in double.                                                        */

static void tap_axis(float coord, int size_img, int size_grid, int* i0, int* i1, double* a) {
  float pitch = (float)size_img / (float)size_grid;
  float q = coord / pitch;
  float g = q - 0.5f;
  g = fminf(fmaxf(g, 0.0f), (float)(size_grid - 1));
  float fl = floorf(g);
  *i0 = (int)fl;
  *i1 = (*i0 + 1 < size_grid) ? *i0 + 1 : size_grid - 1;
  *a = (double)g - (double)fl;
}

static void sample_bilinear(const void* feat_v, int dtype, int Hf, int Wf, int D, int H, int W,
                            float u, float v, double* out /* [D], accumulated into */) {
  int x0, x1, y0, y1;
  double ax, ay;
  tap_axis(u, W, Wf, &x0, &x1, &ax);
  tap_axis(v, H, Hf, &y0, &y1, &ay);
  int64_t o00 = ((int64_t)y0 * Wf + x0) * D, o01 = ((int64_t)y0 * Wf + x1) * D;
  int64_t o10 = ((int64_t)y1 * Wf + x0) * D, o11 = ((int64_t)y1 * Wf + x1) * D;
  for (int c = 0; c < D; ++c) {
    double top = (1.0 - ax) * feat_at(feat_v, dtype, o00 + c) + ax * feat_at(feat_v, dtype, o01 + c);
    double bot = (1.0 - ax) * feat_at(feat_v, dtype, o10 + c) + ax * feat_at(feat_v, dtype, o11 + c);
    out[c] += (1.0 - ay) * top + ay * bot;
  }
}

static int64_t elt_bytes(int dtype) { return dtype == ORC_F32 ? 4 : 2; }

/* ---------------------------------------------------------------- exported: single-point helpers */

/* Projects one point with one camera: fp32 chain into uvz32[3], double into uvz64[3]. */
int orc_project_point(const float* cam, const float* xyz, float* uvz32, double* uvz64) {
  if (!cam || !xyz) return -1;
  if (uvz32) project_f32(cam, xyz, &uvz32[0], &uvz32[1], &uvz32[2]);
  if (uvz64) project_f64(cam, xyz, &uvz64[0], &uvz64[1], &uvz64[2]);
  return 0;
}

/* Bilinear sample of one view's map at image location (u, v); out[D] is overwritten. */
int orc_sample_bilinear(const void* feat_v, int dtype, int Hf, int Wf, int D, int H, int W,
                        float u, float v, double* out) {
  if (!feat_v || !out) return -1;
  if (dtype < 0 || dtype > 2 || Hf < 1 || Wf < 1 || D < 1 || H < 1 || W < 1) return -2;
  for (int c = 0; c < D; ++c) out[c] = 0.0;
  sample_bilinear(feat_v, dtype, Hf, Wf, D, H, W, u, v, out);
  return 0;
}

int orc_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Objects are CSR ranges: points pt_offsets[b]..pt_offsets[b+1] see views
 * view_offsets[b]..view_offsets[b+1].  NULL offsets with B == 1 = one object.     */
static int check_csr(int64_t N, int n_views, const int64_t* pt_offsets, const int32_t* view_offsets, int B) {
  if (B < 1) return -2;
  if (!pt_offsets || !view_offsets) return (B == 1 && !pt_offsets && !view_offsets) ? 0 : -1;
  if (pt_offsets[0] != 0 || pt_offsets[B] != N || view_offsets[0] != 0 || view_offsets[B] != n_views) return -2;
  for (int b = 0; b < B; ++b)
    if (pt_offsets[b + 1] < pt_offsets[b] || view_offsets[b + 1] < view_offsets[b]) return -2;
  return 0;
}

/* ---------------------------------------------------------------- exported: a1 + a2
 * vis[i * vis_pitch + j] = M_vis(x_i, j-th view of the point's object), 0 beyond the
 * object's view count; count[i] = sum_j vis; uvz (optional) [N][vis_pitch][3] fp32;
 * diag (optional) [N][vis_pitch] ORC_DIAG_* bits.                                  */
int orc_project_visibility(const float* cam, const float* depth, int n_views, int H, int W,
                           float tau, float z_near, unsigned flags,
                           const float* xyz, int64_t N, const int64_t* pt_offsets,
                           const int32_t* view_offsets, int B, int vis_pitch,
                           uint8_t* vis, int32_t* count, float* uvz, uint8_t* diag) {
  if (!cam || !xyz || !vis || !count) return -1;
  if (!(flags & ORC_FLAG_FRUSTUM_ONLY) && !depth) return -1;
  if (N < 0 || n_views < 1 || H < 1 || W < 1) return -2;
  int rc = check_csr(N, n_views, pt_offsets, view_offsets, B);
  if (rc) return rc;
  int frustum_only = (flags & ORC_FLAG_FRUSTUM_ONLY) != 0;
  for (int b = 0; b < B; ++b) {
    int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    int v0 = view_offsets ? view_offsets[b] : 0, v1 = view_offsets ? view_offsets[b + 1] : n_views;
    if (v1 - v0 > vis_pitch) return -2;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = p0; i < p1; ++i) {
      int32_t c = 0;
      for (int j = 0; j < vis_pitch; ++j) {
        int64_t o = i * vis_pitch + j;
        vis[o] = 0;
        if (diag) diag[o] = 0;
        if (uvz) uvz[3 * o] = uvz[3 * o + 1] = uvz[3 * o + 2] = 0.0f;
        if (j >= v1 - v0) continue;
        const float* cm = cam + (int64_t)(v0 + j) * 16;
        const float* dv = depth ? depth + (int64_t)(v0 + j) * H * W : NULL;
        float u, v, z;
        project_f32(cm, xyz + 3 * i, &u, &v, &z);
        int m = visible_f32(dv, H, W, tau, z_near, frustum_only, u, v, z);
        vis[o] = (uint8_t)m;
        c += m;
        if (uvz) { uvz[3 * o] = u; uvz[3 * o + 1] = v; uvz[3 * o + 2] = z; }
        if (diag) diag[o] = (uint8_t)diag_flags(cm, dv, H, W, tau, z_near, frustum_only, xyz + 3 * i, u, v, z, m);
      }
      count[i] = c;
    }
  }
  return 0;
}

/* ---------------------------------------------------------------- exported: a1..a4, Eq. 2
 * fused[i] = sum_v M_vis F_v(pi(x_i,v)) / sum_v M_vis, then divided by
 * max(||.||_2, norm_eps) unless ORC_FLAG_MEAN_ONLY.  No visible view: zeros.
 * With sel_mask the weight of a pair is sel_mask[i][v] (the top-k views of Sec. 3.2.2, fused by
 * averaging as in Sec. 3.2.3) instead of M_vis.                                    */
int orc_fuse_features(const float* cam, const float* depth, const void* feat, int feat_dtype,
                      int n_views, int H, int W, int Hf, int Wf, int D,
                      float tau, float z_near, float norm_eps, unsigned flags,
                      const float* xyz, int64_t N, const int64_t* pt_offsets,
                      const int32_t* view_offsets, int B,
                      const uint8_t* sel_mask /* [N][mask_pitch] or NULL */, int mask_pitch,
                      double* fused /* [N][D] */, int32_t* count /* [N] or NULL */) {
  if (!cam || !feat || !xyz || !fused) return -1;
  if (!(flags & ORC_FLAG_FRUSTUM_ONLY) && !depth && !sel_mask) return -1;
  if (N < 0 || n_views < 1 || H < 1 || W < 1 || Hf < 1 || Wf < 1 || D < 1) return -2;
  if (feat_dtype < 0 || feat_dtype > 2) return -3;
  int rc = check_csr(N, n_views, pt_offsets, view_offsets, B);
  if (rc) return rc;
  int frustum_only = (flags & ORC_FLAG_FRUSTUM_ONLY) != 0;
  int64_t view_bytes = (int64_t)Hf * Wf * D * elt_bytes(feat_dtype);
  for (int b = 0; b < B; ++b) {
    int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    int v0 = view_offsets ? view_offsets[b] : 0, v1 = view_offsets ? view_offsets[b + 1] : n_views;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = p0; i < p1; ++i) {
      double* acc = fused + i * D;
      for (int c = 0; c < D; ++c) acc[c] = 0.0;
      int32_t n = 0;
      for (int vw = v0; vw < v1; ++vw) {
        const float* dv = depth ? depth + (int64_t)vw * H * W : NULL;
        float u, v, z;
        project_f32(cam + (int64_t)vw * 16, xyz + 3 * i, &u, &v, &z);
        if (sel_mask) {
          /* Sec. 3.2.3: the mean runs over the views selected for the point (given), not over all visible ones;
             a selected pair must still lie in front of the camera and inside the image */
          if (!sel_mask[i * mask_pitch + (vw - v0)] || !visible_f32(NULL, H, W, tau, z_near, 1, u, v, z)) continue;
        } else if (!visible_f32(dv, H, W, tau, z_near, frustum_only, u, v, z)) {
          continue;
        }
        sample_bilinear((const char*)feat + (int64_t)vw * view_bytes, feat_dtype, Hf, Wf, D, H, W, u, v, acc);
        ++n;
      }
      if (count) count[i] = n;
      if (n == 0) continue;
      for (int c = 0; c < D; ++c) acc[c] /= (double)n;
      if (flags & ORC_FLAG_MEAN_ONLY) continue;
      double ss = 0.0;
      for (int c = 0; c < D; ++c) ss += acc[c] * acc[c];
      double nrm = sqrt(ss);
      if (nrm < (double)norm_eps) nrm = (double)norm_eps;
      for (int c = 0; c < D; ++c) acc[c] /= nrm;
    }
  }
  return 0;
}

/* ---------------------------------------------------------------- exported: a5 + a6, Eq. 4
 * scores[i][k] = <fused_i, temb_k>; prop[i][p] = sum_k softmax_k(scores/T) y[k][p];
 * label[i] = argmax_k scores (lowest index on ties); margin[i] = top1 - top2.
 * unseen_zero: Eq. 2 is 0 / 0 for a point that no view sees and the fused row is taken as all zero; Eq. 4 then gives
 * the plain mean of y (all similarities equal).  With unseen_zero != 0 such a row (every element exactly zero) gets
 * zero properties instead: the other reading of "no observation".  Scores and label are the same either way.   */
int orc_material_scores(const double* fused, int64_t N, int D, const float* temb, int K,
                        const float* y, int P, float T, int unseen_zero,
                        double* scores, double* prop, int32_t* label, double* margin) {
  if (!fused || !temb || !scores) return -1;
  if (N < 0 || D < 1 || K < 1 || P < 0 || (prop && (!y || P < 1)) || !(T > 0.0f)) return -2;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t i = 0; i < N; ++i) {
    const double* f = fused + i * D;
    double* w = scores + i * K;
    for (int k = 0; k < K; ++k) {
      double s = 0.0;
      for (int c = 0; c < D; ++c) s += f[c] * (double)temb[(int64_t)k * D + c];
      w[k] = s;
    }
    int best = 0;
    for (int k = 1; k < K; ++k) if (w[k] > w[best]) best = k;
    if (label) label[i] = best;
    if (margin) {
      double second = -INFINITY;
      for (int k = 0; k < K; ++k) if (k != best && w[k] > second) second = w[k];
      margin[i] = (K > 1) ? w[best] - second : INFINITY;
    }
    if (prop) {
      double den = 0.0;
      for (int p = 0; p < P; ++p) prop[i * P + p] = 0.0;
      for (int k = 0; k < K; ++k) {
        double e = exp((w[k] - w[best]) / (double)T);
        den += e;
        for (int p = 0; p < P; ++p) prop[i * P + p] += e * (double)y[(int64_t)k * P + p];
      }
      for (int p = 0; p < P; ++p) prop[i * P + p] /= den;
      if (unseen_zero) {
        int all_zero = 1;
        for (int c = 0; c < D; ++c) if (f[c] != 0.0) { all_zero = 0; break; }
        if (all_zero) for (int p = 0; p < P; ++p) prop[i * P + p] = 0.0;
      }
    }
  }
  return 0;
}

/* ---------------------------------------------------------------- exported: a7
 * A point is used when count == NULL or count[i] > 0.
 * G == 0 (point-volume mode): mass[b] = sum_i used_i * prop[i][p_index] * vol_i,
 *   vol_i = vol[i] if vol != NULL else vol_uniform.
 * G > 0 (grid mode): object b has a cube grid of G^3 voxels of side grid_h[b] with
 *   lower corner grid_lo[b]; a point's voxel index per axis is
 *   clamp(floor((x - lo) * (1/h)), 0, G-1) taken in fp32 (1/h one fp32 division);
 *   mass[b] = h^3 * sum over occupied voxels of the mean property of its points.  */
int orc_property_integrate(const double* prop, int64_t N, int P, int p_index,
                           const int32_t* count, const float* vol, float vol_uniform,
                           const int64_t* pt_offsets, int B,
                           const float* xyz, const float* grid_lo, const float* grid_h, int G,
                           double* mass, int64_t* n_used) {
  if (!prop || !mass) return -1;
  if (N < 0 || P < 1 || p_index < 0 || p_index >= P || B < 1 || G < 0) return -2;
  if (G > 0 && (!xyz || !grid_lo || !grid_h)) return -1;
  if (!pt_offsets && B != 1) return -1;
  if (pt_offsets) {
    if (pt_offsets[0] != 0 || pt_offsets[B] != N) return -2;
    for (int b = 0; b < B; ++b) if (pt_offsets[b + 1] < pt_offsets[b]) return -2;
  }
  double* vsum = NULL;
  int32_t* vcnt = NULL;
  int64_t G3 = (int64_t)G * G * G;
  if (G > 0) {
    vsum = (double*)malloc(sizeof(double) * (size_t)G3);
    vcnt = (int32_t*)malloc(sizeof(int32_t) * (size_t)G3);
    if (!vsum || !vcnt) { free(vsum); free(vcnt); return -5; }
  }
  for (int b = 0; b < B; ++b) {
    int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    double m = 0.0;
    int64_t used = 0;
    if (G == 0) {
      for (int64_t i = p0; i < p1; ++i) {
        if (count && count[i] <= 0) continue;
        double v = vol ? (double)vol[i] : (double)vol_uniform;
        m += prop[i * P + p_index] * v;
        ++used;
      }
    } else {
      for (int64_t j = 0; j < G3; ++j) { vsum[j] = 0.0; vcnt[j] = 0; }
      float h = grid_h[b];
      float inv_h = 1.0f / h;
      for (int64_t i = p0; i < p1; ++i) {
        if (count && count[i] <= 0) continue;
        int64_t idx = 0;
        for (int a = 2; a >= 0; --a) {              /* idx = (iz*G + iy)*G + ix */
          float t = xyz[3 * i + a] - grid_lo[3 * b + a];
          float s = t * inv_h;
          float fl = floorf(s);
          int q = (fl >= (float)(G - 1)) ? G - 1 : ((fl > 0.0f) ? (int)fl : 0);
          idx = idx * G + q;
        }
        vsum[idx] += prop[i * P + p_index];
        vcnt[idx] += 1;
        ++used;
      }
      double tot = 0.0;
      for (int64_t j = 0; j < G3; ++j) if (vcnt[j] > 0) tot += vsum[j] / (double)vcnt[j];
      m = tot * (double)h * (double)h * (double)h;
    }
    mass[b] = m;
    if (n_used) n_used[b] = used;
  }
  free(vsum);
  free(vcnt);
  return 0;
}

/* ---------------------------------------------------------------- exported: Eq. 5 (densification)
 * For every query q: phi_j = cosine similarity of fq[q] and fs[j] (0 when either vector is zero); N_k(q) =
 * the k sources with the largest phi (of equal values the lower index first; k is cut to Ns);
 *     wq[q][m] = sum_{j in N_k} phi_j ws[j][m] / sum_{j in N_k} phi_j
 * (when |sum phi| < 1e-12 the vector of the nearest source is taken).  Then Eq. 4 on wq[q]:
 * prop[q][p] = sum_m softmax_m(wq/T) y[m][p]; label = argmax_m wq (lowest index on ties).
 * nn_idx / nn_sim [Nq][k]: the neighbours in selection order (-1 / 0 beyond Ns); gap[q] = phi of the k-th
 * neighbour minus the largest phi left out (+inf when nothing is left out).                              */
int orc_knn_densify(const double* fq, int64_t Nq, const double* fs, int Ns, int D, const double* ws, int K, int k,
                    const float* y, int P, float T,
                    double* wq, double* prop, int32_t* label, int32_t* nn_idx, double* nn_sim, double* gap) {
  if (!fq || !fs || !ws || !wq) return -1;
  if (Nq < 0 || Ns < 1 || D < 1 || K < 1 || k < 1 || P < 0 || (prop && (!y || P < 1)) || !(T > 0.0f)) return -2;
  const int ke = k < Ns ? k : Ns;
  double* snorm = (double*)malloc(sizeof(double) * (size_t)Ns);
  if (!snorm) return -3;
  for (int j = 0; j < Ns; ++j) {
    double ss = 0.0;
    for (int c = 0; c < D; ++c) ss += fs[(int64_t)j * D + c] * fs[(int64_t)j * D + c];
    snorm[j] = sqrt(ss);
  }
#pragma omp parallel
  {
    double* phi = (double*)malloc(sizeof(double) * (size_t)Ns);
    char* taken = (char*)malloc((size_t)Ns);
#pragma omp for schedule(dynamic, 64)
    for (int64_t q = 0; q < Nq; ++q) {
      const double* f = fq + q * D;
      double qq = 0.0;
      for (int c = 0; c < D; ++c) qq += f[c] * f[c];
      const double qn = sqrt(qq);
      for (int j = 0; j < Ns; ++j) {
        double dot = 0.0;
        for (int c = 0; c < D; ++c) dot += f[c] * fs[(int64_t)j * D + c];
        phi[j] = (qn > 0.0 && snorm[j] > 0.0) ? dot / (qn * snorm[j]) : 0.0;
        taken[j] = 0;
      }
      double* w = wq + q * K;
      for (int m = 0; m < K; ++m) w[m] = 0.0;
      double den = 0.0;
      int first = -1;
      double kth = 0.0;
      for (int t = 0; t < k; ++t) {
        int best = -1;
        if (t < ke) {
          for (int j = 0; j < Ns; ++j)
            if (!taken[j] && (best < 0 || phi[j] > phi[best])) best = j;   /* ascending j: the lower index wins ties */
          taken[best] = 1;
          if (t == 0) first = best;
          kth = phi[best];
          den += phi[best];
          for (int m = 0; m < K; ++m) w[m] += phi[best] * ws[(int64_t)best * K + m];
        }
        if (nn_idx) nn_idx[q * k + t] = best;
        if (nn_sim) nn_sim[q * k + t] = best >= 0 ? phi[best] : 0.0;
      }
      if (gap) {
        double rest = -INFINITY;
        for (int j = 0; j < Ns; ++j) if (!taken[j] && phi[j] > rest) rest = phi[j];
        gap[q] = (ke < Ns) ? kth - rest : INFINITY;
      }
      if (fabs(den) < 1e-12) {
        for (int m = 0; m < K; ++m) w[m] = ws[(int64_t)first * K + m];
      } else {
        for (int m = 0; m < K; ++m) w[m] /= den;
      }
      int top = 0;
      for (int m = 1; m < K; ++m) if (w[m] > w[top]) top = m;
      if (label) label[q] = top;
      if (prop) {
        double z = 0.0;
        for (int p = 0; p < P; ++p) prop[q * P + p] = 0.0;
        for (int m = 0; m < K; ++m) {
          const double e = exp((w[m] - w[top]) / (double)T);
          z += e;
          for (int p = 0; p < P; ++p) prop[q * P + p] += e * (double)y[(int64_t)m * P + p];
        }
        for (int p = 0; p < P; ++p) prop[q * P + p] /= z;
      }
    }
    free(phi);
    free(taken);
  }
  free(snorm);
  return 0;
}

/* ---------------------------------------------------------------- exported: Sec. 3.4.2, thickness-based integration
 * Every point s of object b is the centre of a voxel b_adap x b_adap x theta:
 *     A_bar  = (L * scale_factor)^2 / N_b          (area one point stands for; N_b = all points of the object)
 *     b_adap = sqrt(A_bar)
 *     zeta(s) = [ sum_k exp(omega_k[s] / T) y_k theta_k / sum_k exp(omega_k[s] / T) ] * b_adap^2 * lambda
 * and the object-level value is the sum of zeta over the object's used points (count == NULL or count[i] > 0).
 * L: box_len[b] when given, else the longest side of the axis-aligned bounding box of all the object's points.
 * The centre of mass named in Sec. 2.1 / 3.4 is the zeta-weighted mean position, sum zeta x / sum zeta
 * (zero when the sum is zero).
 * omega [N][K], y_col [K] (the property column: density for mass), theta [K], xyz [N][3].
 * Outputs: zeta [N] or NULL (0 for unused points), total [B], com [B][3] or NULL, b_adap [B] or NULL,
 * n_used [B] or NULL.                                                                                   */
int orc_thickness_integrate(const double* omega, int64_t N, int K, const float* y_col, const float* theta,
                            const float* xyz, const int32_t* count, const int64_t* pt_offsets, int B,
                            const float* box_len, float T, float lambda, float scale_factor,
                            double* zeta, double* total, double* com, double* b_adap, int64_t* n_used) {
  if (!omega || !y_col || !theta || !xyz || !total) return -1;
  if (N < 0 || K < 1 || B < 1 || !(T > 0.0f)) return -2;
  if (!pt_offsets && B != 1) return -1;
  if (pt_offsets) {
    if (pt_offsets[0] != 0 || pt_offsets[B] != N) return -2;
    for (int b = 0; b < B; ++b) if (pt_offsets[b + 1] < pt_offsets[b]) return -2;
  }
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    double L = 0.0;
    if (box_len) {
      L = (double)box_len[b];
    } else {
      for (int a = 0; a < 3; ++a) {
        double lo = INFINITY, hi = -INFINITY;
        for (int64_t i = p0; i < p1; ++i) {
          const double v = (double)xyz[3 * i + a];
          if (v < lo) lo = v;
          if (v > hi) hi = v;
        }
        if (p1 > p0 && hi - lo > L) L = hi - lo;
      }
    }
    const double side = L * (double)scale_factor;
    const double area = p1 > p0 ? side * side / (double)(p1 - p0) : 0.0;
    double m = 0.0, mx[3] = {0.0, 0.0, 0.0};
    int64_t used = 0;
    for (int64_t i = p0; i < p1; ++i) {
      if (zeta) zeta[i] = 0.0;
      if (count && count[i] <= 0) continue;
      const double* w = omega + i * K;
      double top = w[0];
      for (int k = 1; k < K; ++k) if (w[k] > top) top = w[k];
      double num = 0.0, den = 0.0;
      for (int k = 0; k < K; ++k) {
        const double e = exp((w[k] - top) / (double)T);     /* the common factor exp(top / T) cancels */
        num += e * (double)y_col[k] * (double)theta[k];
        den += e;
      }
      const double z = num / den * area * (double)lambda;
      if (zeta) zeta[i] = z;
      m += z;
      for (int a = 0; a < 3; ++a) mx[a] += z * (double)xyz[3 * i + a];
      ++used;
    }
    total[b] = m;
    if (com) for (int a = 0; a < 3; ++a) com[3 * b + a] = m != 0.0 ? mx[a] / m : 0.0;
    if (b_adap) b_adap[b] = sqrt(area);
    if (n_used) n_used[b] = used;
  }
  return 0;
}

/* ---------------------------------------------------------------- exported: Sec. 3.2.2, view importance-based filtering
 * For every visible pair (Eq. 1, the fp32 decision above):
 *     S_dist  = 1 / (1 + z),  z = depth of the point in the camera frame
 *     S_angle = max(0, v . (-n)),  v = unit vector from the camera centre C = -R^T t to the point, n = the
 *               point's unit normal (as given, oriented outward)
 *     S_total = S_dist * S_angle
 * and the k visible views with the largest S_total are kept (of equal scores the lower view index first).
 * Scores are double.  sel_view / sel_score [N][k]: the kept views (index within the object) in rank order,
 * -1 / 0 beyond the number of visible views; sel_mask [N][mask_pitch]: 1 for kept pairs; n_sel [N];
 * gap [N]: S_total of the last kept view minus the largest S_total left out (+inf when nothing is left out);
 * score_all [N][mask_pitch] or NULL: S_total of every visible pair, -1 for the others.                 */
int orc_select_views(const float* cam, const float* depth, int n_views, int H, int W, float tau, float z_near,
                     unsigned flags, const float* xyz, const float* normals, int64_t N,
                     const int64_t* pt_offsets, const int32_t* view_offsets, int B, int k, int mask_pitch,
                     int32_t* sel_view, double* sel_score, uint8_t* sel_mask, int32_t* n_sel, double* gap,
                     double* score_all) {
  if (!cam || !xyz || !normals || !sel_view) return -1;
  if (!(flags & ORC_FLAG_FRUSTUM_ONLY) && !depth) return -1;
  if (N < 0 || n_views < 1 || H < 1 || W < 1 || k < 1) return -2;
  int rc = check_csr(N, n_views, pt_offsets, view_offsets, B);
  if (rc) return rc;
  const int frustum_only = (flags & ORC_FLAG_FRUSTUM_ONLY) != 0;
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    const int v0 = view_offsets ? view_offsets[b] : 0, v1 = view_offsets ? view_offsets[b + 1] : n_views;
    const int nv = v1 - v0;
    if ((sel_mask || score_all) && mask_pitch < nv) return -2;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = p0; i < p1; ++i) {
      double* S = (double*)malloc(sizeof(double) * (size_t)(nv > 0 ? nv : 1));
      char* taken = (char*)calloc((size_t)(nv > 0 ? nv : 1), 1);
      const double x[3] = {xyz[3 * i], xyz[3 * i + 1], xyz[3 * i + 2]};
      const double n[3] = {normals[3 * i], normals[3 * i + 1], normals[3 * i + 2]};
      for (int j = 0; j < nv; ++j) {
        const float* cm = cam + (int64_t)(v0 + j) * 16;
        const float* dv = depth ? depth + (int64_t)(v0 + j) * H * W : NULL;
        float u, v, z;
        project_f32(cm, xyz + 3 * i, &u, &v, &z);
        S[j] = -1.0;                                        /* not visible */
        if (!visible_f32(dv, H, W, tau, z_near, frustum_only, u, v, z)) continue;
        double ud, vd, zd;
        project_f64(cm, xyz + 3 * i, &ud, &vd, &zd);
        double ray[3], len = 0.0;
        for (int a = 0; a < 3; ++a) {                       /* C = -R^T t: C_a = -sum_r R[r][a] t[r] */
          const double c = -((double)cm[a] * cm[9] + (double)cm[3 + a] * cm[10] + (double)cm[6 + a] * cm[11]);
          ray[a] = x[a] - c;
          len += ray[a] * ray[a];
        }
        len = sqrt(len);
        double dot = 0.0;
        for (int a = 0; a < 3; ++a) dot += ray[a] / len * (-n[a]);
        S[j] = (1.0 / (1.0 + zd)) * (dot > 0.0 ? dot : 0.0);
      }
      if (sel_mask) for (int j = 0; j < mask_pitch; ++j) sel_mask[i * mask_pitch + j] = 0;
      if (score_all) for (int j = 0; j < mask_pitch; ++j) score_all[i * mask_pitch + j] = j < nv ? S[j] : -1.0;
      int kept = 0;
      double last = 0.0;
      for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int j = 0; j < nv; ++j)
          if (!taken[j] && S[j] >= 0.0 && (best < 0 || S[j] > S[best])) best = j;
        sel_view[i * k + r] = best;
        if (sel_score) sel_score[i * k + r] = best >= 0 ? S[best] : 0.0;
        if (best < 0) continue;
        taken[best] = 1;
        last = S[best];
        ++kept;
        if (sel_mask) sel_mask[i * mask_pitch + best] = 1;
      }
      if (n_sel) n_sel[i] = kept;
      if (gap) {
        double rest = -INFINITY;
        for (int j = 0; j < nv; ++j) if (!taken[j] && S[j] >= 0.0 && S[j] > rest) rest = S[j];
        gap[i] = (kept > 0 && rest > -INFINITY) ? last - rest : INFINITY;
      }
      free(S);
      free(taken);
    }
  }
  return 0;
}

/* ---------------------------------------------------------------- exported: Sec. 3.2.1, adaptive sampling
 * Voxel size from the volume of the boundary box and the wanted number of points,
 *     s_voxel = cbrt(V_bound / N_target),
 * then standard voxel down-sampling: the box is cut into cubes of side s_voxel and every occupied cube is
 * replaced by the mean position of its points.
 * Decision arithmetic (fp32, so that an fp32 implementation bins every point alike): extents e = hi - lo,
 * s = (float)cbrt((double)e_x * e_y * e_z / N_target); a flat box (volume 0) takes the longest extent in place of
 * the cube root of the volume, s = e_max / cbrt(N_target), and a box of one point s = 1; cubes per axis
 * n = floor(e / s) + 1; a point's cube per axis clamp(floor((x - lo) / s), 0, n - 1).                     */
int orc_voxel_grid(const float* box_lo, const float* box_hi, int n_target, float* s_voxel, int32_t* dims) {
  if (!box_lo || !box_hi || !s_voxel || !dims) return -1;
  if (n_target < 1) return -2;
  float e[3], emax = 0.0f;
  for (int a = 0; a < 3; ++a) {
    e[a] = box_hi[a] - box_lo[a];
    if (!(e[a] >= 0.0f)) return -2;
    if (e[a] > emax) emax = e[a];
  }
  float s = (float)cbrt((double)e[0] * (double)e[1] * (double)e[2] / (double)n_target);
  if (!(s > 0.0f)) s = (float)((double)emax / cbrt((double)n_target));
  if (!(s > 0.0f)) s = 1.0f;
  *s_voxel = s;
  for (int a = 0; a < 3; ++a) {
    float q = floorf(e[a] / s);
    if (q > 2.0e9f) return -7;
    dims[a] = (int32_t)q + 1;
  }
  return 0;
}

/* out_xyz / out_count: the occupied cubes of object 0 in the order of their index (z * ny + y) * nx + x, then those
 * of object 1, ...; out_offsets [B+1] their ranges; voxel_of_point [N]: position of the point's cube in that list.
 * Returns the number of occupied cubes through *n_out; out arrays hold out_capacity entries (cubes beyond are
 * counted but not written).                                                                              */
int orc_voxel_downsample(const float* xyz, int64_t N, const int64_t* pt_offsets, int B, const float* box_lo,
                         const float* box_hi, int n_target, double* out_xyz, int32_t* out_count, int64_t out_capacity,
                         int64_t* out_offsets, int64_t* voxel_of_point) {
  if (!xyz || !box_lo || !box_hi || !out_xyz || !out_offsets) return -1;
  if (N < 0 || B < 1 || n_target < 1) return -2;
  if (!pt_offsets && B != 1) return -1;
  int64_t total = 0;
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : N;
    float s;
    int32_t d[3];
    int rc = orc_voxel_grid(box_lo + 3 * b, box_hi + 3 * b, n_target, &s, d);
    if (rc) return rc;
    const int64_t cells = (int64_t)d[0] * d[1] * d[2];
    double* sum = (double*)calloc((size_t)cells * 3, sizeof(double));
    int32_t* cnt = (int32_t*)calloc((size_t)cells, sizeof(int32_t));
    int64_t* slot = (int64_t*)malloc((size_t)cells * sizeof(int64_t));
    int64_t* cell_of = (int64_t*)malloc((size_t)(p1 > p0 ? p1 - p0 : 1) * sizeof(int64_t));
    if (!sum || !cnt || !slot || !cell_of) { free(sum); free(cnt); free(slot); free(cell_of); return -5; }
    for (int64_t i = p0; i < p1; ++i) {
      int64_t idx = 0;
      for (int a = 2; a >= 0; --a) {
        float t = xyz[3 * i + a] - box_lo[3 * b + a];
        float fl = floorf(t / s);
        int q = (fl >= (float)(d[a] - 1)) ? d[a] - 1 : ((fl > 0.0f) ? (int)fl : 0);
        idx = idx * d[a] + q;
      }
      cell_of[i - p0] = idx;
      for (int a = 0; a < 3; ++a) sum[3 * idx + a] += (double)xyz[3 * i + a];
      cnt[idx] += 1;
    }
    out_offsets[b] = total;
    for (int64_t c = 0; c < cells; ++c) {
      slot[c] = -1;
      if (cnt[c] == 0) continue;
      slot[c] = total;
      if (total < out_capacity) {
        for (int a = 0; a < 3; ++a) out_xyz[3 * total + a] = sum[3 * c + a] / (double)cnt[c];
        if (out_count) out_count[total] = cnt[c];
      }
      ++total;
    }
    if (voxel_of_point) for (int64_t i = p0; i < p1; ++i) voxel_of_point[i] = slot[cell_of[i - p0]];
    free(sum); free(cnt); free(slot); free(cell_of);
  }
  out_offsets[B] = total;
  return 0;
}

/* ---------------------------------------------------------------- exported: Sec. 3.2.3, multi-scale patches
 * For point s, each of its kept views v (sel_view, index within the object; -1: none) and each scale l (side of
 * the square in pixels, e.g. 20, 40, 60): the patch P_v^(l)(s) is the l x l square of view v's image centred at the
 * projection pi(s, v) = (u, v), resampled to R x R for the encoder.  The image is read as a continuous field
 * (bilinear between pixel centres at integer + 0.5, the border pixel repeated outside the image); output pixel
 * (i, j) samples it at
 *     x = u - l/2 + (j + 0.5) l / R,   y = v - l/2 + (i + 0.5) l / R
 * and is stored channel-first as (value / 255 - mean[c]) * inv_std[c].
 * images [n_views][H][W][3] uint8; out [M][k][L][3][R][R] double; valid [M][k] or NULL.
 * The projection is the fp32 chain of project_f32; everything after it is double.                          */
int orc_patch_batch(const float* cam, int n_views, int H, int W, const uint8_t* images, const float* xyz, int64_t M,
                    const int64_t* pt_offsets, const int32_t* view_offsets, int B, const int32_t* sel_view, int k,
                    const float* scales, int L, int R, const float* mean, const float* inv_std, double* out,
                    uint8_t* valid) {
  if (!cam || !images || !xyz || !sel_view || !scales || !out) return -1;
  if (M < 0 || n_views < 1 || H < 1 || W < 1 || k < 1 || L < 1 || R < 1) return -2;
  int rc = check_csr(M, n_views, pt_offsets, view_offsets, B);
  if (rc) return rc;
  const int64_t plane = (int64_t)R * R;
  for (int b = 0; b < B; ++b) {
    const int64_t p0 = pt_offsets ? pt_offsets[b] : 0, p1 = pt_offsets ? pt_offsets[b + 1] : M;
    const int v0 = view_offsets ? view_offsets[b] : 0, v1 = view_offsets ? view_offsets[b + 1] : n_views;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t s = p0; s < p1; ++s) {
      for (int r = 0; r < k; ++r) {
        const int sv = sel_view[s * k + r];
        double* o = out + (s * k + r) * (int64_t)L * 3 * plane;
        const int ok = sv >= 0 && sv < v1 - v0;
        if (valid) valid[s * k + r] = (uint8_t)ok;
        if (!ok) {
          for (int64_t e = 0; e < (int64_t)L * 3 * plane; ++e) o[e] = 0.0;
          continue;
        }
        const uint8_t* img = images + (int64_t)(v0 + sv) * H * W * 3;
        float uf, vf, zf;
        project_f32(cam + (int64_t)(v0 + sv) * 16, xyz + 3 * s, &uf, &vf, &zf);
        for (int l = 0; l < L; ++l) {
          const double side = (double)scales[l];
          for (int i = 0; i < R; ++i) {
            for (int j = 0; j < R; ++j) {
              const double x = (double)uf - 0.5 * side + ((double)j + 0.5) * side / (double)R;
              const double y = (double)vf - 0.5 * side + ((double)i + 0.5) * side / (double)R;
              /* pixel centres at integer + 0.5: texel coordinates g = x - 0.5, clamped to the image */
              double gx = x - 0.5, gy = y - 0.5;
              if (gx < 0.0) gx = 0.0;
              if (gx > (double)(W - 1)) gx = (double)(W - 1);
              if (gy < 0.0) gy = 0.0;
              if (gy > (double)(H - 1)) gy = (double)(H - 1);
              const int x0 = (int)floor(gx), y0 = (int)floor(gy);
              const int x1 = x0 + 1 < W ? x0 + 1 : W - 1, y1 = y0 + 1 < H ? y0 + 1 : H - 1;
              const double ax = gx - (double)x0, ay = gy - (double)y0;
              for (int c = 0; c < 3; ++c) {
                const double t00 = img[((int64_t)y0 * W + x0) * 3 + c], t01 = img[((int64_t)y0 * W + x1) * 3 + c];
                const double t10 = img[((int64_t)y1 * W + x0) * 3 + c], t11 = img[((int64_t)y1 * W + x1) * 3 + c];
                const double val = (1.0 - ay) * ((1.0 - ax) * t00 + ax * t01) + ay * ((1.0 - ax) * t10 + ax * t11);
                const double mu = mean ? (double)mean[c] : 0.0, is = inv_std ? (double)inv_std[c] : 1.0;
                o[((int64_t)l * 3 + c) * plane + (int64_t)i * R + j] = (val / 255.0 - mu) * is;
              }
            }
          }
        }
      }
    }
  }
  return 0;
}
