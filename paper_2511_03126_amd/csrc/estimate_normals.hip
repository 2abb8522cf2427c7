// aura_estimate_normals: the normals of the sampled points, which the view importance score needs (Sec. 3.2.2, first
// step of the view filtering).
//
// For every sampled point q: the k points of the object's cloud nearest to q, the plane through them (eigenvector of
// the smallest eigenvalue of their covariance), turned to point away from the object's centre.
//
// One workgroup per query.  Which points are nearest is decided on the fp32 distance d = (dx dx + dy dy) + dz dz
// (every operation rounded, no contraction), of equal distances the lower index first.
//
// Usual path (k up to 256), one sweep over the cloud:
//   1. an upper bound of the k-th smallest distance that is exact by construction: the k-th smallest distance among
//      every stride-th point (at most 16384 of them; the k-th smallest of a subset can only be larger);
//   2. one sweep over the whole cloud collects the points within that bound (about k * stride of them) in LDS;
//   3. among those, the k-th smallest distance by a radix select over the bit pattern of d (non-negative floats order
//      like their bits: histograms of the next 11 / 11 / 10 bits among the candidates left) and, when more points share
//      that distance than are still needed, the same select over their indices;
//   4. the selected points in index order: r and r r^T (r = p - q, exact in fp64) summed in that order by one
//      thread, then the covariance and a cyclic Jacobi iteration on the 3 x 3 matrix.
// General path (larger k, or more candidates than the LDS list holds, e.g. thousands of points at one distance): the
// radix select over the whole cloud (three sweeps), then one sweep for the sums.
// The queries of a call run side by side; the cloud comes from L2 (a few MB) or the last-level cache.
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

constexpr int kNrmBlock = 1024;   // a sweep over the cloud is shared by 16 waves
constexpr int kNrmBins = 2048;
constexpr int kNrmSub = 16384;    // points of the strided subset that bounds the k-th distance
constexpr int kNrmCand = 4096;    // candidates the LDS list holds
constexpr int kNrmSel = 256;      // largest k of the one-sweep path

struct NrmObjDev {
  long long pt_begin;
  int n_pts;
  int q_begin;
  int n_q;
  float centre[3];
};

struct NrmTable {
  NrmObjDev o[kMaxObjPerLaunch];
};

struct NrmArgs {
  const float* xyz;
  const float* queries;
  int k;
  float* normals;   // [M][3]
  float* evals;     // [M][3] or nullptr: eigenvalues of the covariance, ascending
};

__device__ __forceinline__ uint32_t dist_bits(const float* __restrict__ p, float qx, float qy, float qz) {
#pragma clang fp contract(off)
  const float dx = p[0] - qx, dy = p[1] - qy, dz = p[2] - qz;
  float t = dx * dx + dy * dy;
  t = t + dz * dz;
  return __float_as_uint(t);
}

// Among the elements i of [0, n) with eligible(i), the `want`-th smallest key(i) (want >= 1, at most the number of
// eligible elements): returns the key; *n_equal = how many eligible elements have that key, *need = how many of them
// belong to the `want` smallest.  All threads of the workgroup call it and get the same answer.
template <typename Key, typename Eligible>
__device__ uint32_t radix_select(int n, int want, Key key, Eligible eligible, uint32_t* s_hist, int* s_pick, int* n_equal,
                                 int* need) {
  uint32_t prefix = 0, mask = 0;
  int remaining = want;
  const int shifts[3] = {21, 10, 0}, widths[3] = {11, 11, 10};
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = shifts[pass], nb = 1 << widths[pass];
    for (int b = threadIdx.x; b < kNrmBins; b += kNrmBlock) s_hist[b] = 0;
    __syncthreads();
    // four points per thread and trip, so that their reads are in flight together
    for (int i0 = threadIdx.x; i0 < n; i0 += 4 * kNrmBlock) {
      uint32_t kv[4];
      bool cand[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = i0 + e * kNrmBlock;
        cand[e] = i < n && eligible(i);
        kv[e] = cand[e] ? key(i) : 0u;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (cand[e] && (kv[e] & mask) == prefix) atomicAdd(&s_hist[(kv[e] >> shift) & (uint32_t)(nb - 1)], 1u);
    }
    __syncthreads();
    // the bin that holds the remaining-th candidate: thread t sums its kPer consecutive bins, a scan over the threads
    // finds the thread, which then walks its bins
    constexpr int kPer = kNrmBins / kNrmBlock;
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < kPer; ++e) mine += s_hist[threadIdx.x * kPer + e];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    uint32_t inc = mine;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const uint32_t up = __shfl_up(inc, o, kWave);
      if (lane >= o) inc += up;
    }
    __shared__ uint32_t s_wave[kNrmBlock / kWave];
    if (lane == kWave - 1) s_wave[wave] = inc;
    __syncthreads();
    uint32_t before = inc - mine;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    if ((uint32_t)remaining > before && (uint32_t)remaining <= before + mine) {   // exactly one thread
      uint32_t run = before;
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        const uint32_t c = s_hist[threadIdx.x * kPer + e];
        if ((uint32_t)remaining > run && (uint32_t)remaining <= run + c) {
          s_pick[0] = threadIdx.x * kPer + e;
          s_pick[1] = (int)run;
          s_pick[2] = (int)c;
        }
        run += c;
      }
    }
    __syncthreads();
    prefix |= (uint32_t)s_pick[0] << shift;
    mask |= (uint32_t)(nb - 1) << shift;
    remaining -= s_pick[1];
    *n_equal = s_pick[2];
    __syncthreads();   // s_pick and s_hist are free again
  }
  *need = remaining;
  return prefix;
}

__device__ __forceinline__ double nrm_block_sum(double v, double* sh) {
  v = wave_sum(v);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < kNrmBlock / kWave; ++w) t += sh[w];
  return t;
}

// Eigenvalues (ascending in w) and the eigenvector of the smallest one of the symmetric matrix
// [a00 a01 a02; a01 a11 a12; a02 a12 a22], by cyclic Jacobi rotations.
__device__ void smallest_eigenvector(const double (&c)[6], double (&w)[3], double (&n)[3]) {
  double a[3][3] = {{c[0], c[1], c[2]}, {c[1], c[3], c[4]}, {c[2], c[4], c[5]}};
  double v[3][3] = {{1, 0, 0}, {0, 1, 0}, {0, 0, 1}};
  for (int sweep = 0; sweep < 24; ++sweep) {
    const double off = fabs(a[0][1]) + fabs(a[0][2]) + fabs(a[1][2]);
    const double diag = fabs(a[0][0]) + fabs(a[1][1]) + fabs(a[2][2]);
    if (off <= 1e-300 || off <= 1e-17 * diag) break;
    for (int p = 0; p < 2; ++p) {
      for (int q = p + 1; q < 3; ++q) {
        if (a[p][q] == 0.0) continue;
        const double theta = (a[q][q] - a[p][p]) / (2.0 * a[p][q]);
        const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
        const double cs = 1.0 / sqrt(t * t + 1.0), sn = t * cs;
        for (int r = 0; r < 3; ++r) {   // A <- A J
          const double arp = a[r][p], arq = a[r][q];
          a[r][p] = cs * arp - sn * arq;
          a[r][q] = sn * arp + cs * arq;
        }
        for (int r = 0; r < 3; ++r) {   // A <- J^T A
          const double apr = a[p][r], aqr = a[q][r];
          a[p][r] = cs * apr - sn * aqr;
          a[q][r] = sn * apr + cs * aqr;
        }
        for (int r = 0; r < 3; ++r) {   // V <- V J
          const double vrp = v[r][p], vrq = v[r][q];
          v[r][p] = cs * vrp - sn * vrq;
          v[r][q] = sn * vrp + cs * vrq;
        }
      }
    }
  }
  int order[3] = {0, 1, 2};
  for (int i = 0; i < 2; ++i)
    for (int j = 0; j < 2 - i; ++j)
      if (a[order[j]][order[j]] > a[order[j + 1]][order[j + 1]]) {
        const int t = order[j];
        order[j] = order[j + 1];
        order[j + 1] = t;
      }
  for (int i = 0; i < 3; ++i) w[i] = a[order[i]][order[i]];
  const double len = sqrt(v[0][order[0]] * v[0][order[0]] + v[1][order[0]] * v[1][order[0]] + v[2][order[0]] * v[2][order[0]]);
  for (int r = 0; r < 3; ++r) n[r] = v[r][order[0]] / len;
}

// From the sums of r and r r^T over the kk selected points to the stored normal (one thread).
__device__ void finish_normal(const NrmArgs& a, const NrmObjDev& ob, long long m, float qx, float qy, float qz, int kk,
                              const double (&s1)[3], const double (&s2)[6]) {
  const double inv = 1.0 / (double)kk;
  const double mx = s1[0] * inv, my = s1[1] * inv, mz = s1[2] * inv;
  const double cov[6] = {s2[0] * inv - mx * mx, s2[1] * inv - mx * my, s2[2] * inv - mx * mz,
                         s2[3] * inv - my * my, s2[4] * inv - my * mz, s2[5] * inv - mz * mz};
  double w[3], nv[3];
  smallest_eigenvector(cov, w, nv);
  const double ox = (double)qx - (double)ob.centre[0], oy = (double)qy - (double)ob.centre[1], oz = (double)qz - (double)ob.centre[2];
  const double sgn = nv[0] * ox + nv[1] * oy + nv[2] * oz < 0.0 ? -1.0 : 1.0;
  for (int c = 0; c < 3; ++c) {
    a.normals[3 * m + c] = (float)(sgn * nv[c]);
    if (a.evals) a.evals[3 * m + c] = (float)w[c];
  }
}

__global__ __launch_bounds__(kNrmBlock) void k_estimate_normals(NrmArgs a, NrmTable tab) {
  __shared__ uint32_t s_hist[kNrmBins];
  __shared__ int s_pick[3];
  __shared__ double s_red[kNrmBlock / kWave];
  const NrmObjDev ob = tab.o[blockIdx.y];
  if ((int)blockIdx.x >= ob.n_q) return;
  const long long m = ob.q_begin + blockIdx.x;
  const float qx = a.queries[3 * m], qy = a.queries[3 * m + 1], qz = a.queries[3 * m + 2];
  const float* __restrict__ pts = a.xyz + 3 * ob.pt_begin;
  const int n = ob.n_pts;
  const int kk = a.k < n ? a.k : n;
  if (kk == 0) {   // an object without points
    if (threadIdx.x < 3) {
      a.normals[3 * m + threadIdx.x] = 0.0f;
      if (a.evals) a.evals[3 * m + threadIdx.x] = 0.0f;
    }
    return;
  }
  auto dist = [&](int i) { return dist_bits(pts + 3 * (long long)i, qx, qy, qz); };
  int n_equal, need;
  if (kk <= kNrmSel) {
    __shared__ uint32_t s_cd[kNrmCand];   // candidates: distance bits ...
    __shared__ int s_ci[kNrmCand];        // ... and point index
    __shared__ int s_cn, s_ns;
    __shared__ int s_sel[kNrmSel];        // the k selected points, unordered, then in index order
    __shared__ float s_pt[kNrmSel][3];
    const int stride = (n + kNrmSub - 1) / kNrmSub;
    const int m_sub = (n + stride - 1) / stride;   // >= kk: kk <= n, and kk <= 256 < 16384 where stride > 1
    const uint32_t bound = radix_select(m_sub, kk, [&](int j) { return dist(j * stride); }, [](int) { return true; }, s_hist,
                                        s_pick, &n_equal, &need);
    if (threadIdx.x == 0) { s_cn = 0; s_ns = 0; }
    __syncthreads();
    for (int i0 = threadIdx.x; i0 < n; i0 += 8 * kNrmBlock) {   // eight points per thread and trip: reads in flight together
      uint32_t d[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = dist(min(i0 + e * kNrmBlock, n - 1));
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i = i0 + e * kNrmBlock;
        if (i < n && d[e] <= bound) {
          const int pos = atomicAdd(&s_cn, 1);
          if (pos < kNrmCand) { s_cd[pos] = d[e]; s_ci[pos] = i; }
        }
      }
    }
    __syncthreads();
    const int cn = s_cn;
    if (cn <= kNrmCand) {   // uniform; otherwise the general path below
      const uint32_t tau = radix_select(cn, kk, [&](int j) { return s_cd[j]; }, [](int) { return true; }, s_hist, s_pick,
                                        &n_equal, &need);
      int last_idx = 0x7fffffff;   // points at distance tau are taken up to this index
      if (need < n_equal) {
        int e2, n2;
        last_idx = (int)radix_select(cn, need, [&](int j) { return (uint32_t)s_ci[j]; }, [&](int j) { return s_cd[j] == tau; },
                                     s_hist, s_pick, &e2, &n2);
      }
      for (int j = threadIdx.x; j < cn; j += kNrmBlock)
        if (s_cd[j] < tau || (s_cd[j] == tau && s_ci[j] <= last_idx)) s_sel[atomicAdd(&s_ns, 1)] = s_ci[j];   // exactly kk
      __syncthreads();
      // index order: the rank of a selected point is the number of selected points before it
      int mine = -1, rank = 0;
      if ((int)threadIdx.x < kk) {
        mine = s_sel[threadIdx.x];
        for (int j = 0; j < kk; ++j) rank += s_sel[j] < mine ? 1 : 0;
      }
      __syncthreads();
      if (mine >= 0) {
        const float* __restrict__ pm = pts + 3 * (long long)mine;
        s_pt[rank][0] = pm[0]; s_pt[rank][1] = pm[1]; s_pt[rank][2] = pm[2];
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        double s1[3] = {0, 0, 0}, s2[6] = {0, 0, 0, 0, 0, 0};
        for (int j = 0; j < kk; ++j) {
          const double rx = (double)s_pt[j][0] - (double)qx, ry = (double)s_pt[j][1] - (double)qy, rz = (double)s_pt[j][2] - (double)qz;
          s1[0] += rx; s1[1] += ry; s1[2] += rz;
          s2[0] += rx * rx; s2[1] += rx * ry; s2[2] += rx * rz;
          s2[3] += ry * ry; s2[4] += ry * rz; s2[5] += rz * rz;
        }
        finish_normal(a, ob, m, qx, qy, qz, kk, s1, s2);
      }
      return;
    }
  }
  const uint32_t tau = radix_select(n, kk, dist, [](int) { return true; }, s_hist, s_pick, &n_equal, &need);
  int last_idx = 0x7fffffff;   // points at distance tau are taken up to this index
  if (need < n_equal) {
    int e2, n2;
    last_idx = (int)radix_select(n, need, [](int i) { return (uint32_t)i; }, [&](int i) { return dist(i) == tau; }, s_hist,
                                 s_pick, &e2, &n2);
  }
  double s1[3] = {0, 0, 0}, s2[6] = {0, 0, 0, 0, 0, 0};
  for (int i0 = threadIdx.x; i0 < n; i0 += 4 * kNrmBlock) {
    float px[4], py[4], pz[4];
    bool in[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = min(i0 + e * kNrmBlock, n - 1);
      const float* __restrict__ p = pts + 3 * (long long)i;
      px[e] = p[0]; py[e] = p[1]; pz[e] = p[2];
      in[e] = i0 + e * kNrmBlock < n;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = i0 + e * kNrmBlock;
      const float pe[3] = {px[e], py[e], pz[e]};
      const uint32_t d = dist_bits(pe, qx, qy, qz);
      if (in[e] && (d < tau || (d == tau && i <= last_idx))) {
        const double rx = (double)px[e] - (double)qx, ry = (double)py[e] - (double)qy, rz = (double)pz[e] - (double)qz;
        s1[0] += rx; s1[1] += ry; s1[2] += rz;
        s2[0] += rx * rx; s2[1] += rx * ry; s2[2] += rx * rz;
        s2[3] += ry * ry; s2[4] += ry * rz; s2[5] += rz * rz;
      }
    }
  }
#pragma unroll
  for (int c = 0; c < 3; ++c) s1[c] = nrm_block_sum(s1[c], s_red);
#pragma unroll
  for (int c = 0; c < 6; ++c) s2[c] = nrm_block_sum(s2[c], s_red);
  if (threadIdx.x == 0) finish_normal(a, ob, m, qx, qy, qz, kk, s1, s2);
}

hipError_t launch_estimate_normals(const float* xyz, const float* queries, const NrmObj* objs, int n_obj, int k,
                                   float* normals, float* evals, hipStream_t stream) {
  NrmTable tab{};
  int max_q = 0;
  for (int b = 0; b < n_obj; ++b) {
    NrmObjDev& d = tab.o[b];
    d.pt_begin = objs[b].pt_begin; d.n_pts = objs[b].n_pts; d.q_begin = objs[b].q_begin; d.n_q = objs[b].n_q;
    for (int c = 0; c < 3; ++c) d.centre[c] = objs[b].centre[c];
    max_q = d.n_q > max_q ? d.n_q : max_q;
  }
  if (max_q == 0) return hipSuccess;
  NrmArgs a{xyz, queries, k, normals, evals};
  hipLaunchKernelGGL(k_estimate_normals, dim3(max_q, n_obj), dim3(kNrmBlock), 0, stream, a, tab);
  return hipGetLastError();
}

}  // namespace aura
