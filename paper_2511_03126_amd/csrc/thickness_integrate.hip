// aura_thickness_integrate: Sec. 3.4.2, thickness-based voxel integration, and the centre of mass.
//
// Every point s of an object stands for a voxel b_adap x b_adap x theta_k:
//     A_bar = (L * scale_factor)^2 / N_b,  b_adap = sqrt(A_bar),
//     zeta(s) = sum_k softmax_k(omega_k[s] / T) y_k theta_k * b_adap^2 * lambda,
// the object-level value is the sum of zeta over the object's used points and the centre of mass is the
// zeta-weighted mean position.  L is the longest side of the bounding box of all the object's points (or a length
// given by the caller), N_b the number of all its points.
//
// Three launches, all bound by launch latency for the sizes of one object (a few bytes per point besides the
// score rows, which are read once):
//   k_thick_box     per slice of points: minima and maxima of the coordinates       (skipped when L is given)
//   k_thick_points  per slice of points: every workgroup first reduces the slices' boxes of its object (all
//                   workgroups of an object read the same values and find the same L), then one thread per point
//                   walks the point's score row; zeta and zeta * position are summed over the workgroup in fp64
//   k_thick_final   per object: the slices' sums added in a fixed order, so results are reproducible bit for bit
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

constexpr int kThBlock = 256;
constexpr int kThPtsPerBlock = kThBlock;   // slice of points handled by one workgroup: one point per thread
constexpr int kThMaxK = 128;

struct ThickObjDev {
  long long pt_begin;
  int n_pts;
  int slice_begin;   // first slot of this object in the per-slice arrays
  int n_slices;
  float box_len;     // < 0: take the longest side of the bounding box
};

struct ThickTable {
  ThickObjDev o[kMaxObjPerLaunch];
};

struct ThickArgs {
  const float* scores;   // [N][K]
  int K;
  const float* y;        // [K][P]
  int P, p_index;
  const float* theta;    // [K]
  const float* xyz;      // [N][3]
  const int* count;      // [N] or nullptr
  float inv_T, lambda, scale;
  float* zeta;           // [N] or nullptr
  float* box_part;       // [slices][6]: minima, maxima
  double* part;          // [slices][4]: sum zeta, sum zeta x, sum zeta y, sum zeta z
  long long* part_used;  // [slices]
  float* obj_area;       // [B]: A_bar
  int obj_base;
};

__global__ __launch_bounds__(kThBlock) void k_thick_box(ThickArgs a, ThickTable tab) {
  __shared__ float sh[kThBlock / kWave][6];
  const ThickObjDev ob = tab.o[blockIdx.y];
  if ((int)blockIdx.x >= ob.n_slices || ob.box_len >= 0.0f) return;
  const int begin = blockIdx.x * kThPtsPerBlock;
  const int end = min(begin + kThPtsPerBlock, ob.n_pts);
  float lo[3] = {INFINITY, INFINITY, INFINITY}, hi[3] = {-INFINITY, -INFINITY, -INFINITY};
  for (int li = begin + threadIdx.x; li < end; li += kThBlock) {
    const float* p = a.xyz + 3 * (ob.pt_begin + li);
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      lo[c] = fminf(lo[c], p[c]);
      hi[c] = fmaxf(hi[c], p[c]);
    }
  }
#pragma unroll
  for (int c = 0; c < 3; ++c) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
      lo[c] = fminf(lo[c], __shfl_xor(lo[c], o, kWave));
      hi[c] = fmaxf(hi[c], __shfl_xor(hi[c], o, kWave));
    }
  }
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (lane == 0) {
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      sh[wave][c] = lo[c];
      sh[wave][3 + c] = hi[c];
    }
  }
  __syncthreads();
  if (threadIdx.x < 6) {
    float v = sh[0][threadIdx.x];
    for (int w = 1; w < kThBlock / kWave; ++w) v = threadIdx.x < 3 ? fminf(v, sh[w][threadIdx.x]) : fmaxf(v, sh[w][threadIdx.x]);
    a.box_part[(size_t)(ob.slice_begin + blockIdx.x) * 6 + threadIdx.x] = v;
  }
}

// A_bar of an object from its slices' boxes (or the given length); every thread of the workgroup gets the value.
__device__ __forceinline__ float object_area(const ThickArgs& a, const ThickObjDev& ob, float (*sh)[6]) {
#pragma clang fp contract(off)
  float L = ob.box_len;
  if (L < 0.0f) {
    float lo[3] = {INFINITY, INFINITY, INFINITY}, hi[3] = {-INFINITY, -INFINITY, -INFINITY};
    for (int s = threadIdx.x; s < ob.n_slices; s += kThBlock) {
      const float* p = a.box_part + (size_t)(ob.slice_begin + s) * 6;
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        lo[c] = fminf(lo[c], p[c]);
        hi[c] = fmaxf(hi[c], p[3 + c]);
      }
    }
#pragma unroll
    for (int c = 0; c < 3; ++c) {
#pragma unroll
      for (int o = kWave / 2; o > 0; o >>= 1) {
        lo[c] = fminf(lo[c], __shfl_xor(lo[c], o, kWave));
        hi[c] = fmaxf(hi[c], __shfl_xor(hi[c], o, kWave));
      }
    }
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    __syncthreads();
    if (lane == 0) {
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        sh[wave][c] = lo[c];
        sh[wave][3 + c] = hi[c];
      }
    }
    __syncthreads();
    L = 0.0f;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      float l = sh[0][c], h = sh[0][3 + c];
      for (int w = 1; w < kThBlock / kWave; ++w) {
        l = fminf(l, sh[w][c]);
        h = fmaxf(h, sh[w][3 + c]);
      }
      L = fmaxf(L, h - l);
    }
  }
  const float side = L * a.scale;
  return ob.n_pts > 0 ? side * side / (float)ob.n_pts : 0.0f;
}

__device__ __forceinline__ double thick_block_sum(double v, double* sh) {
  v = wave_sum(v);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < kThBlock / kWave; ++w) t += sh[w];
  return t;
}

// One point per thread.  The score row is walked twice (largest score, then the two sums of the softmax); the second
// walk finds the row in the vector cache.  Rows of K % 4 == 0 scores are read 16 bytes at a time.
template <bool VEC4>
__device__ __forceinline__ float softmax_weighted(const float* __restrict__ row, int K, const float* s_yt, float inv_T) {
  float top = -INFINITY, num = 0.0f, den = 0.0f;
  if constexpr (VEC4) {
    typedef float th_f32x4 __attribute__((ext_vector_type(4)));
    const th_f32x4* __restrict__ r4 = reinterpret_cast<const th_f32x4*>(row);
#pragma unroll 8
    for (int q = 0; q < K / 4; ++q) {
      const th_f32x4 w = r4[q];
      top = fmaxf(fmaxf(top, fmaxf(w[0], w[1])), fmaxf(w[2], w[3]));
    }
#pragma unroll 8
    for (int q = 0; q < K / 4; ++q) {
      const th_f32x4 w = r4[q];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float ex = expf((w[e] - top) * inv_T);
        num = __builtin_fmaf(ex, s_yt[4 * q + e], num);
        den += ex;
      }
    }
  } else {
#pragma unroll 8
    for (int k = 0; k < K; ++k) top = fmaxf(top, row[k]);
#pragma unroll 8
    for (int k = 0; k < K; ++k) {
      const float ex = expf((row[k] - top) * inv_T);
      num = __builtin_fmaf(ex, s_yt[k], num);
      den += ex;
    }
  }
  return num / den;
}

template <bool VEC4>
__global__ __launch_bounds__(kThBlock) void k_thick_points(ThickArgs a, ThickTable tab) {
  __shared__ float s_box[kThBlock / kWave][6];
  __shared__ double s_red[kThBlock / kWave];
  __shared__ float s_yt[kThMaxK];
  const ThickObjDev ob = tab.o[blockIdx.y];
  if ((int)blockIdx.x >= ob.n_slices) return;
  const int K = a.K;
  for (int k = threadIdx.x; k < K; k += kThBlock) s_yt[k] = a.y[(size_t)k * a.P + a.p_index] * a.theta[k];
  const float area = object_area(a, ob, s_box);   // has barriers: s_yt is visible after it ...
  __syncthreads();                                // ... also when the length was given
  if (blockIdx.x == 0 && threadIdx.x == 0) a.obj_area[a.obj_base + blockIdx.y] = area;
  const float coef = area * a.lambda;

  double m = 0.0, mx = 0.0, my = 0.0, mz = 0.0, used = 0.0;
  const int li = blockIdx.x * kThPtsPerBlock + threadIdx.x;
  if (li < ob.n_pts) {
    const long long i = ob.pt_begin + li;
    const bool use = !a.count || a.count[i] > 0;
    float z = 0.0f;
    if (use) {
      z = softmax_weighted<VEC4>(a.scores + i * K, K, s_yt, a.inv_T) * coef;
      const float* p = a.xyz + 3 * i;
      m = (double)z;
      mx = (double)z * (double)p[0];
      my = (double)z * (double)p[1];
      mz = (double)z * (double)p[2];
      used = 1.0;
    }
    if (a.zeta) a.zeta[i] = z;
  }
  m = thick_block_sum(m, s_red);
  mx = thick_block_sum(mx, s_red);
  my = thick_block_sum(my, s_red);
  mz = thick_block_sum(mz, s_red);
  used = thick_block_sum(used, s_red);   // at most 256: exact
  if (threadIdx.x == 0) {
    double* out = a.part + (size_t)(ob.slice_begin + blockIdx.x) * 4;
    out[0] = m; out[1] = mx; out[2] = my; out[3] = mz;
    a.part_used[ob.slice_begin + blockIdx.x] = (long long)used;
  }
}

__global__ __launch_bounds__(kThBlock) void k_thick_final(ThickArgs a, ThickTable tab, float* total, float* com, float* b_adap,
                                                          long long* n_used) {
  __shared__ double s_red[kThBlock / kWave];
  const ThickObjDev ob = tab.o[blockIdx.x];
  double s[4] = {0.0, 0.0, 0.0, 0.0}, used = 0.0;
  for (int j = threadIdx.x; j < ob.n_slices; j += kThBlock) {
    const double* p = a.part + (size_t)(ob.slice_begin + j) * 4;
#pragma unroll
    for (int c = 0; c < 4; ++c) s[c] += p[c];
    used += (double)a.part_used[ob.slice_begin + j];       // below 2^31 in total: exact
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) s[c] = thick_block_sum(s[c], s_red);
  used = thick_block_sum(used, s_red);
  if (threadIdx.x == 0) {
    const int b = a.obj_base + blockIdx.x;
    total[b] = (float)s[0];
    if (com) {
#pragma unroll
      for (int c = 0; c < 3; ++c) com[3 * b + c] = s[0] != 0.0 ? (float)(s[1 + c] / s[0]) : 0.0f;
    }
    if (b_adap) b_adap[b] = ob.n_slices > 0 ? sqrtf(a.obj_area[b]) : 0.0f;
    if (n_used) n_used[b] = (long long)used;
  }
}

// ---------------------------------------------------------------- host side

static size_t th_align256(size_t x) { return (x + 255) & ~(size_t)255; }
static long long th_slices(long long n) { return (n + kThPtsPerBlock - 1) / kThPtsPerBlock; }
static long long th_max_slices(long long N, int B) { return th_slices(N) + B; }   // every object adds at most one partly filled slice

bool thickness_supported(int K) { return K >= 1 && K <= kThMaxK; }

size_t thickness_workspace_bytes(long long N, int B) {
  const size_t nsl = (size_t)th_max_slices(N, B);
  return th_align256(nsl * 6 * sizeof(float)) + th_align256(nsl * 4 * sizeof(double)) + th_align256(nsl * sizeof(long long)) +
         th_align256((size_t)B * sizeof(float));
}

hipError_t launch_thickness_integrate(const float* scores, int K, const float* y, int P, int p_index, const float* theta,
                                      const float* xyz, const int* count, const ThickObj* objs, int B, float temperature,
                                      float lambda, float scale_factor, float* zeta, float* total, float* com,
                                      float* b_adap, long long* n_used, void* workspace, hipStream_t stream) {
  long long N = 0;
  for (int b = 0; b < B; ++b) N += objs[b].n_pts;
  const size_t nsl = (size_t)th_max_slices(N, B);
  char* ws = static_cast<char*>(workspace);
  ThickArgs a{};
  a.scores = scores; a.K = K; a.y = y; a.P = P; a.p_index = p_index; a.theta = theta; a.xyz = xyz; a.count = count;
  a.inv_T = 1.0f / temperature; a.lambda = lambda; a.scale = scale_factor; a.zeta = zeta;
  size_t off = 0;
  a.box_part = reinterpret_cast<float*>(ws + off);      off += th_align256(nsl * 6 * sizeof(float));
  a.part = reinterpret_cast<double*>(ws + off);         off += th_align256(nsl * 4 * sizeof(double));
  a.part_used = reinterpret_cast<long long*>(ws + off); off += th_align256(nsl * sizeof(long long));
  a.obj_area = reinterpret_cast<float*>(ws + off);

  const int n_chunks = (B + kMaxObjPerLaunch - 1) / kMaxObjPerLaunch;
  int cursor = 0;
  for (int c = 0; c < n_chunks; ++c) {
    ThickTable tab{};
    const int obj_base = c * kMaxObjPerLaunch;
    const int n_obj = B - obj_base < kMaxObjPerLaunch ? B - obj_base : kMaxObjPerLaunch;
    int max_slices = 0;
    bool need_box = false;
    for (int t = 0; t < n_obj; ++t) {
      const ThickObj& o = objs[obj_base + t];
      ThickObjDev& d = tab.o[t];
      d.pt_begin = o.pt_begin; d.n_pts = o.n_pts; d.box_len = o.box_len;
      d.n_slices = (int)th_slices(o.n_pts);
      d.slice_begin = cursor;
      cursor += d.n_slices;
      max_slices = d.n_slices > max_slices ? d.n_slices : max_slices;
      need_box = need_box || (o.box_len < 0.0f && o.n_pts > 0);
    }
    a.obj_base = obj_base;
    const dim3 block(kThBlock), grid(max_slices > 0 ? max_slices : 1, n_obj);
    if (max_slices > 0) {
      if (need_box) hipLaunchKernelGGL(k_thick_box, grid, block, 0, stream, a, tab);
      // 16-byte reads need rows that start on 16 bytes
      if (K % 4 == 0 && (reinterpret_cast<uintptr_t>(scores) & 15) == 0)
        hipLaunchKernelGGL((k_thick_points<true>), grid, block, 0, stream, a, tab);
      else
        hipLaunchKernelGGL((k_thick_points<false>), grid, block, 0, stream, a, tab);
    }
    hipLaunchKernelGGL(k_thick_final, dim3(n_obj), block, 0, stream, a, tab, total, com, b_adap, n_used);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace aura
