// aura_property_integrate: Sec. 3.4.2, integration of a property over voxels.
//
// Point-volume mode: mass[b] = sum_i used_i * prop_i * vol_i.  Each workgroup sums a fixed slice of
// an object's points in fp64 (fp32 products), a second kernel adds the slices in a fixed order.
//
// Grid mode: points are binned into the object's G^3 voxels; the per-voxel property sums are
// accumulated EXACTLY as 64-bit fixed-point integers (integer atomics commute, so the result does
// not depend on the order in which the atomics land), the per-voxel means are then summed in
// fp64 in a fixed order.  The fixed-point scale is chosen from the largest |prop| of the call so
// that no sum can overflow.
//
// All traffic is a few bytes per point plus one sweep over the voxel arrays: the call is a small
// fraction of the fusion pass and is bound by launch latency for small inputs.  Grid mode is four
// launches: (1) zero the voxel arrays and take the largest |prop| per slice of points, (2) bin,
// (3) per-voxel means summed per slice of voxels, (4) the slices added in a fixed order; with more than 1024 slices of
// points a one-workgroup launch between (1) and (2) reduces the per-slice maxima to one word.
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

constexpr int kMassBlock = 256;
constexpr int kMassPtsPerBlock = 512;    // slice of points summed by one workgroup
constexpr int kVoxPerBlock = 2048;       // slice of voxels summed by one workgroup
constexpr int kAbsmaxPerGroup = 1024;    // up to this many slices of points every workgroup takes their maximum itself

struct MassObjDev {
  long long pt_begin;
  int n_pts;
  float lo[3];
  float h;
  int slice_begin;   // first partial-sum slot of this object
  int n_slices;
};

struct MassTable {
  MassObjDev o[kMaxObjPerLaunch];
};

struct MassArgs {
  const float* prop;
  int P, p_index;
  const int* count;
  const float* vol;
  float vol_uniform;
  const float* xyz;
  int G;
  double* part_sum;        // [total slices]
  long long* part_used;    // [total slices]
  unsigned* absmax_part;   // [slices of points]: largest |prop| bits per slice (grid mode)
  int n_absmax;            // number of valid entries of absmax_part
  const unsigned* absmax_call;   // their maximum, where k_mass_absmax has taken it (many slices); else null
  long long* vox_sum;      // [B * G^3] fixed point
  int* vox_cnt;            // [B * G^3]
  int obj_base;            // index of the table's first object within the call
  int n_points_bits;       // ceil(log2(N + 1)), for the fixed-point scale
};

__device__ __forceinline__ double block_sum(double v, double* sh) {
  v = wave_sum(v);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < kMassBlock / kWave; ++w) t += sh[w];
  return t;
}

__device__ __forceinline__ long long block_sum(long long v, long long* sh) {
  v = wave_sum(v);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  long long t = 0;
  for (int w = 0; w < kMassBlock / kWave; ++w) t += sh[w];
  return t;
}

// ---------------------------------------------------------------- point-volume mode

__global__ __launch_bounds__(kMassBlock) void k_mass_points(MassArgs a, MassTable tab) {
  __shared__ double shd[kMassBlock / kWave];
  __shared__ long long shl[kMassBlock / kWave];
  const MassObjDev ob = tab.o[blockIdx.y];
  if ((int)blockIdx.x >= ob.n_slices) return;
  const int begin = blockIdx.x * kMassPtsPerBlock;
  const int end = min(begin + kMassPtsPerBlock, ob.n_pts);
  double s = 0.0;
  long long used = 0;
  for (int li = begin + threadIdx.x; li < end; li += kMassBlock) {
    const long long i = ob.pt_begin + li;
    if (a.count && a.count[i] <= 0) continue;
    const float v = a.vol ? a.vol[i] : a.vol_uniform;
    s += (double)(a.prop[i * a.P + a.p_index] * v);
    ++used;
  }
  s = block_sum(s, shd);
  used = block_sum(used, shl);
  if (threadIdx.x == 0) {
    a.part_sum[ob.slice_begin + blockIdx.x] = s;
    a.part_used[ob.slice_begin + blockIdx.x] = used;
  }
}

// ---------------------------------------------------------------- grid mode

// Launch 1 of grid mode.  Every workgroup zeroes its share of the voxel arrays;
// workgroup (x, object) with x below the object's slice count also writes the largest |prop| over the used
// points of its slice, as the bit pattern of a non-negative float (monotone), into its slot.
typedef uint32_t mass_u32x4 __attribute__((ext_vector_type(4)));
typedef int mass_i32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kMassBlock) void k_mass_prepare(MassArgs a, MassTable tab, uint32_t* zero_from, long long zero_vecs) {
  {
    mass_u32x4* __restrict__ z = reinterpret_cast<mass_u32x4*>(zero_from);   // 256-byte aligned, a multiple of 256 bytes
    const long long nthreads = (long long)gridDim.x * gridDim.y * kMassBlock;
    long long i = ((long long)blockIdx.y * gridDim.x + blockIdx.x) * kMassBlock + threadIdx.x;
    for (; i < zero_vecs; i += nthreads) z[i] = mass_u32x4{0u, 0u, 0u, 0u};
  }
  __shared__ unsigned shm[kMassBlock / kWave];
  const MassObjDev ob = tab.o[blockIdx.y];
  if ((int)blockIdx.x >= ob.n_slices) return;
  const int begin = blockIdx.x * kMassPtsPerBlock;
  const int end = min(begin + kMassPtsPerBlock, ob.n_pts);
  unsigned m = 0;
  for (int li = begin + threadIdx.x; li < end; li += kMassBlock) {
    const long long i = ob.pt_begin + li;
    if (a.count && a.count[i] <= 0) continue;
    m = max(m, __float_as_uint(fabsf(a.prop[i * a.P + a.p_index])));
  }
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o, kWave));
  if (threadIdx.x % kWave == 0) shm[threadIdx.x / kWave] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kMassBlock / kWave; ++w) m = max(m, shm[w]);
    a.absmax_part[ob.slice_begin + blockIdx.x] = m;
  }
}

// Largest |prop| of the call from the per-slice maxima.  With few slices every workgroup that needs the scale takes it
// from them; with many, k_mass_absmax has done that once (64 objects of 100 000 points: 12 544 slices, which each of
// the 12 544 + 8 192 workgroups of the two kernels below read in 49 trips - more than their own work).
__device__ __forceinline__ unsigned call_absmax(const MassArgs& a, unsigned* sh) {
  if (a.absmax_call) return *a.absmax_call;   // the same for every thread of the launch
  unsigned m = 0;
  for (int j = threadIdx.x; j < a.n_absmax; j += kMassBlock) m = max(m, a.absmax_part[j]);
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o, kWave));
  if (threadIdx.x % kWave == 0) sh[threadIdx.x / kWave] = m;
  __syncthreads();
  m = sh[0];
#pragma unroll
  for (int w = 1; w < kMassBlock / kWave; ++w) m = max(m, sh[w]);
  return m;
}

constexpr int kAbsmaxBlock = 1024;

__global__ __launch_bounds__(kAbsmaxBlock) void k_mass_absmax(MassArgs a, unsigned* out) {
  __shared__ unsigned shm[kAbsmaxBlock / kWave];
  unsigned m = 0;
  const int n4 = a.n_absmax / 4;   // the array starts on a 256-byte boundary
  const mass_u32x4* __restrict__ p4 = reinterpret_cast<const mass_u32x4*>(a.absmax_part);
  for (int j = threadIdx.x; j < n4; j += kAbsmaxBlock) {
    const mass_u32x4 v = p4[j];
    m = max(m, max(max(v[0], v[1]), max(v[2], v[3])));
  }
  for (int j = 4 * n4 + threadIdx.x; j < a.n_absmax; j += kAbsmaxBlock) m = max(m, a.absmax_part[j]);
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o, kWave));
  if (threadIdx.x % kWave == 0) shm[threadIdx.x / kWave] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kAbsmaxBlock / kWave; ++w) m = max(m, shm[w]);
    *out = m;
  }
}

// Power-of-two scale s with |x| * 2^s * (number of points) < 2^62 for every used x.
__device__ __forceinline__ int fixed_point_shift(unsigned absmax_bits, int n_points_bits) {
  int e;
  frexpf(__uint_as_float(absmax_bits), &e);   // |x| < 2^e
  if (absmax_bits == 0) e = 0;
  return 62 - e - n_points_bits;
}

__device__ __forceinline__ int voxel_axis(float x, float lo, float inv_h, int G) {
#pragma clang fp contract(off)
  float t = x - lo;
  float s = t * inv_h;
  float fl = floorf(s);
  return (fl >= (float)(G - 1)) ? G - 1 : ((fl > 0.0f) ? (int)fl : 0);
}

__global__ __launch_bounds__(kMassBlock) void k_mass_bin(MassArgs a, MassTable tab) {
  __shared__ unsigned shm[kMassBlock / kWave];
  const MassObjDev ob = tab.o[blockIdx.y];
  if ((int)blockIdx.x >= ob.n_slices) return;
  const int begin = blockIdx.x * kMassPtsPerBlock;
  const int end = min(begin + kMassPtsPerBlock, ob.n_pts);
  const int shift = fixed_point_shift(call_absmax(a, shm), a.n_points_bits);
  const float inv_h = 1.0f / ob.h;
  const long long G = a.G;
  const long long vox0 = (long long)(a.obj_base + blockIdx.y) * G * G * G;
  const int lane = threadIdx.x % kWave;
  for (int l0 = begin; l0 < end; l0 += kMassBlock) {   // uniform trip count: the lanes of a wave exchange values below
    const int li = l0 + threadIdx.x;
    const long long i = ob.pt_begin + min(li, end - 1);
    // all of a point's reads are issued together (the index is clamped: in bounds whether the point is used or not)
    const int cnt = a.count ? a.count[i] : 1;
    const float px = a.xyz[3 * i], py = a.xyz[3 * i + 1], pz = a.xyz[3 * i + 2];
    const float pr = a.prop[i * a.P + a.p_index];
    const bool used = li < end && cnt > 0;
    long long vidx = -1 - lane;   // unused lanes: a voxel id no neighbour shares
    long long q = 0;
    if (used) {
      const int ix = voxel_axis(px, ob.lo[0], inv_h, a.G);
      const int iy = voxel_axis(py, ob.lo[1], inv_h, a.G);
      const int iz = voxel_axis(pz, ob.lo[2], inv_h, a.G);
      vidx = vox0 + ((long long)iz * G + iy) * G + ix;
      q = __double2ll_rn(ldexp((double)pr, shift));
    }
    // Spatially sorted points fall into the same voxel in runs: the lanes of a run add up (integers: the
    // order does not matter) and its last lane issues one pair of atomics for the whole run.
    const long long prev = __shfl_up(vidx, 1, kWave), next = __shfl_down(vidx, 1, kWave);
    const bool head = lane == 0 || prev != vidx, tail = lane == kWave - 1 || next != vidx;
    int start = head ? lane : 0;   // lane of the run's first member
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) start = max(start, __shfl_up(start, o, kWave));
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const long long up = __shfl_up(q, o, kWave);
      if (lane - o >= start) q += up;
    }
    if (used && tail) {
      atomicAdd(reinterpret_cast<unsigned long long*>(a.vox_sum + vidx), (unsigned long long)q);
      atomicAdd(a.vox_cnt + vidx, lane - start + 1);
    }
  }
}

// Launch 3 of grid mode: sum of per-voxel means over one slice of an object's voxels.
__global__ __launch_bounds__(kMassBlock) void k_mass_voxels(MassArgs a, MassTable tab) {
  __shared__ double shd[kMassBlock / kWave];
  __shared__ long long shl[kMassBlock / kWave];
  __shared__ unsigned shm[kMassBlock / kWave];
  const MassObjDev ob = tab.o[blockIdx.y];
  const long long G3 = (long long)a.G * a.G * a.G;
  const long long vox0 = (long long)(a.obj_base + blockIdx.y) * G3;
  const long long begin = (long long)blockIdx.x * kVoxPerBlock;
  const long long end = min(begin + (long long)kVoxPerBlock, G3);
  const int shift = fixed_point_shift(call_absmax(a, shm), a.n_points_bits);
  double s = 0.0;
  long long used = 0;
  // a thread takes four consecutive voxels per trip: their counts in one 16-byte read, the sums of the occupied ones only
  // (the points of a surface occupy a few percent of a 64^3 grid)
  for (long long j = begin + 4 * threadIdx.x; j < end; j += 4 * kMassBlock) {
    const int* __restrict__ cp = a.vox_cnt + vox0 + j;
    int c[4];
    if (j + 4 <= end && (reinterpret_cast<uintptr_t>(cp) & 15) == 0) {
      const mass_i32x4 v = *reinterpret_cast<const mass_i32x4*>(cp);
      c[0] = v[0], c[1] = v[1], c[2] = v[2], c[3] = v[3];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) c[e] = j + e < end ? cp[e] : 0;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (c[e] > 0) {
        s += ldexp((double)a.vox_sum[vox0 + j + e], -shift) / (double)c[e];
        used += c[e];
      }
    }
  }
  s = block_sum(s, shd);
  used = block_sum(used, shl);
  if (threadIdx.x == 0) {
    a.part_sum[ob.slice_begin + blockIdx.x] = s;
    a.part_used[ob.slice_begin + blockIdx.x] = used;
  }
}

// ---------------------------------------------------------------- final fixed-order sum

__global__ __launch_bounds__(kMassBlock) void k_mass_final(MassArgs a, MassTable tab, float* mass, long long* n_used) {
  __shared__ double shd[kMassBlock / kWave];
  __shared__ long long shl[kMassBlock / kWave];
  const MassObjDev ob = tab.o[blockIdx.x];
  double s = 0.0;
  long long used = 0;
  for (int j = threadIdx.x; j < ob.n_slices; j += kMassBlock) {
    s += a.part_sum[ob.slice_begin + j];
    used += a.part_used[ob.slice_begin + j];
  }
  s = block_sum(s, shd);
  used = block_sum(used, shl);
  if (threadIdx.x == 0) {
    if (a.G > 0) s *= (double)ob.h * (double)ob.h * (double)ob.h;
    mass[a.obj_base + blockIdx.x] = (float)s;
    if (n_used) n_used[a.obj_base + blockIdx.x] = used;
  }
}

// ---------------------------------------------------------------- host side

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static long long slices_points(long long n) { return (n + kMassPtsPerBlock - 1) / kMassPtsPerBlock; }
static long long slices_voxels(int G) { return ((long long)G * G * G + kVoxPerBlock - 1) / kVoxPerBlock; }

// Upper bound on partial-sum slots: every object adds at most one partly filled slice.
static long long max_slices(long long N, int B, int G) {
  return G > 0 ? (long long)B * slices_voxels(G) : slices_points(N) + B;
}

size_t integrate_workspace_bytes(long long N, int B, int G) {
  size_t bytes = align256((size_t)max_slices(N, B, G) * sizeof(double));
  bytes += align256((size_t)max_slices(N, B, G) * sizeof(long long));
  if (G > 0) {
    size_t vox = (size_t)B * G * G * G;
    bytes += align256((size_t)(slices_points(N) + B + 1) * sizeof(unsigned));                   // per-slice maxima, their maximum
    bytes += align256(vox * sizeof(long long)) + align256(vox * sizeof(int));
  }
  return bytes;
}

hipError_t launch_property_integrate(const float* prop, int P, int p_index, const int* count, const float* vol,
                                     float vol_uniform, const MassObj* objs, int B, const float* xyz, int G,
                                     float* mass, long long* n_used, void* workspace, hipStream_t stream) {
  long long N = 0;
  for (int b = 0; b < B; ++b) N += objs[b].n_pts;
  char* ws = static_cast<char*>(workspace);
  MassArgs a{};
  a.prop = prop; a.P = P; a.p_index = p_index; a.count = count; a.vol = vol; a.vol_uniform = vol_uniform;
  a.xyz = xyz; a.G = G;
  size_t off = 0;
  const long long nsl = max_slices(N, B, G);
  a.part_sum = reinterpret_cast<double*>(ws + off);     off += align256((size_t)nsl * sizeof(double));
  a.part_used = reinterpret_cast<long long*>(ws + off); off += align256((size_t)nsl * sizeof(long long));
  const size_t vox = G > 0 ? (size_t)B * G * G * G : 0;
  size_t zero_begin = 0, zero_end = 0;   // the voxel sums and the voxel counts must start at zero
  if (G > 0) {
    a.absmax_part = reinterpret_cast<unsigned*>(ws + off); off += align256((size_t)(slices_points(N) + B + 1) * sizeof(unsigned));
    zero_begin = off;
    a.vox_sum = reinterpret_cast<long long*>(ws + off); off += align256(vox * sizeof(long long));
    a.vox_cnt = reinterpret_cast<int*>(ws + off);       off += align256(vox * sizeof(int));
    zero_end = off;
  }
  a.n_points_bits = 1;
  while (a.n_points_bits < 40 && (1ll << a.n_points_bits) <= N) ++a.n_points_bits;
  for (int b = 0; b < B; ++b) a.n_absmax += (int)slices_points(objs[b].n_pts);

  // objects go to the device in tables of kMaxObjPerLaunch; grid mode needs every object's maxima
  // and bins finished before any voxel is read, so the passes run over all tables one after another
  const int n_chunks = (B + kMaxObjPerLaunch - 1) / kMaxObjPerLaunch;
  const int n_passes = G > 0 ? 4 : 2;
  for (int pass = 0; pass < n_passes; ++pass) {
    int pt_cursor = 0, vox_cursor = 0;
    if (G > 0 && pass == 1 && a.n_absmax > kAbsmaxPerGroup) {   // the slot behind the last per-slice maximum
      unsigned* out = a.absmax_part + (slices_points(N) + B);
      hipLaunchKernelGGL(k_mass_absmax, dim3(1), dim3(kAbsmaxBlock), 0, stream, a, out);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      a.absmax_call = out;
    }
    for (int c = 0; c < n_chunks; ++c) {
      MassTable tab{};
      const int obj_base = c * kMaxObjPerLaunch;
      const int n_obj = B - obj_base < kMaxObjPerLaunch ? B - obj_base : kMaxObjPerLaunch;
      const bool by_voxels = G > 0 && pass >= 2;
      int max_pt_slices = 0;
      for (int t = 0; t < n_obj; ++t) {
        const MassObj& o = objs[obj_base + t];
        MassObjDev& d = tab.o[t];
        d.pt_begin = o.pt_begin; d.n_pts = o.n_pts;
        d.lo[0] = o.lo[0]; d.lo[1] = o.lo[1]; d.lo[2] = o.lo[2]; d.h = o.h;
        const int pt_slices = (int)slices_points(o.n_pts);
        max_pt_slices = pt_slices > max_pt_slices ? pt_slices : max_pt_slices;
        d.n_slices = by_voxels ? (int)slices_voxels(G) : pt_slices;
        d.slice_begin = by_voxels ? vox_cursor : pt_cursor;
        pt_cursor += pt_slices;
        vox_cursor += G > 0 ? (int)slices_voxels(G) : 0;
      }
      a.obj_base = obj_base;
      dim3 block(kMassBlock);
      if (G == 0) {
        if (pass == 0) {
          if (max_pt_slices > 0)
            hipLaunchKernelGGL(k_mass_points, dim3(max_pt_slices, n_obj), block, 0, stream, a, tab);
        } else {
          hipLaunchKernelGGL(k_mass_final, dim3(n_obj), block, 0, stream, a, tab, mass, n_used);
        }
      } else if (pass == 0) {
        // the first table's launch also zeroes (16 bytes per thread and trip): give it enough workgroups
        const long long zero_vecs = c == 0 ? (long long)((zero_end - zero_begin) / 16) : 0;
        int gx = max_pt_slices > 1 ? max_pt_slices : 1;
        if (c == 0) {
          const long long want = (zero_vecs / (8 * kMassBlock) + n_obj) / n_obj;
          gx = (int)(want > gx ? (want < 4096 ? want : 4096) : gx);
        }
        hipLaunchKernelGGL(k_mass_prepare, dim3(gx, n_obj), block, 0, stream, a, tab,
                           reinterpret_cast<uint32_t*>(ws + zero_begin), zero_vecs);
      } else if (pass == 1) {
        if (max_pt_slices > 0) hipLaunchKernelGGL(k_mass_bin, dim3(max_pt_slices, n_obj), block, 0, stream, a, tab);
      } else if (pass == 2) {
        hipLaunchKernelGGL(k_mass_voxels, dim3((int)slices_voxels(G), n_obj), block, 0, stream, a, tab);
      } else {
        hipLaunchKernelGGL(k_mass_final, dim3(n_obj), block, 0, stream, a, tab, mass, n_used);
      }
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

}  // namespace aura
