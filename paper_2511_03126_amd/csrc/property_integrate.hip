// aura_property_integrate: Sec. 3.4.2 "voxel integration over volumes".
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
// fraction of the fusion pass and is bound by launch latency for small inputs.
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

constexpr int kMassBlock = 256;
constexpr int kMassPtsPerBlock = 512;    // slice of points summed by one workgroup
constexpr int kVoxPerBlock = 2048;       // slice of voxels summed by one workgroup

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
  unsigned* absmax_bits;   // [1]
  long long* vox_sum;      // [B * G^3] fixed point
  int* vox_cnt;            // [B * G^3]
  int obj_base;            // index of the table's first object within the call
  int n_points_bits;       // ceil(log2(N + 1)), for the fixed-point scale
};

__global__ void k_fill_zero(uint32_t* p, long long n_words) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  long long stride = (long long)gridDim.x * blockDim.x;
  for (; i < n_words; i += stride) p[i] = 0u;
}

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

// Largest |prop| over the used points, as the bit pattern of a non-negative float (monotone).
__global__ __launch_bounds__(kMassBlock) void k_mass_absmax(MassArgs a, MassTable tab) {
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
  if (threadIdx.x % kWave == 0 && m != 0) atomicMax(a.absmax_bits, m);
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
  const MassObjDev ob = tab.o[blockIdx.y];
  if ((int)blockIdx.x >= ob.n_slices) return;
  const int begin = blockIdx.x * kMassPtsPerBlock;
  const int end = min(begin + kMassPtsPerBlock, ob.n_pts);
  const int shift = fixed_point_shift(*a.absmax_bits, a.n_points_bits);
  const float inv_h = 1.0f / ob.h;
  const long long G = a.G;
  const long long vox0 = (long long)(a.obj_base + blockIdx.y) * G * G * G;
  for (int li = begin + threadIdx.x; li < end; li += kMassBlock) {
    const long long i = ob.pt_begin + li;
    if (a.count && a.count[i] <= 0) continue;
    const int ix = voxel_axis(a.xyz[3 * i], ob.lo[0], inv_h, a.G);
    const int iy = voxel_axis(a.xyz[3 * i + 1], ob.lo[1], inv_h, a.G);
    const int iz = voxel_axis(a.xyz[3 * i + 2], ob.lo[2], inv_h, a.G);
    const long long vidx = vox0 + ((long long)iz * G + iy) * G + ix;
    const long long q = __double2ll_rn(ldexp((double)a.prop[i * a.P + a.p_index], shift));
    atomicAdd(reinterpret_cast<unsigned long long*>(a.vox_sum + vidx), (unsigned long long)q);
    atomicAdd(a.vox_cnt + vidx, 1);
  }
}

// Sum of per-voxel means over one slice of an object's voxels.
__global__ __launch_bounds__(kMassBlock) void k_mass_voxels(MassArgs a, MassTable tab) {
  __shared__ double shd[kMassBlock / kWave];
  __shared__ long long shl[kMassBlock / kWave];
  const MassObjDev ob = tab.o[blockIdx.y];
  const long long G3 = (long long)a.G * a.G * a.G;
  const long long vox0 = (long long)(a.obj_base + blockIdx.y) * G3;
  const long long begin = (long long)blockIdx.x * kVoxPerBlock;
  const long long end = min(begin + (long long)kVoxPerBlock, G3);
  const int shift = fixed_point_shift(*a.absmax_bits, a.n_points_bits);
  double s = 0.0;
  long long used = 0;
  for (long long j = begin + threadIdx.x; j < end; j += kMassBlock) {
    const int c = a.vox_cnt[vox0 + j];
    if (c > 0) {
      s += ldexp((double)a.vox_sum[vox0 + j], -shift) / (double)c;
      used += c;
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
  size_t bytes = 256;                                          // absmax word
  bytes += align256((size_t)max_slices(N, B, G) * sizeof(double));
  bytes += align256((size_t)max_slices(N, B, G) * sizeof(long long));
  if (G > 0) {
    size_t vox = (size_t)B * G * G * G;
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
  a.absmax_bits = reinterpret_cast<unsigned*>(ws);
  size_t off = 256;
  const long long nsl = max_slices(N, B, G);
  a.part_sum = reinterpret_cast<double*>(ws + off);     off += align256((size_t)nsl * sizeof(double));
  a.part_used = reinterpret_cast<long long*>(ws + off); off += align256((size_t)nsl * sizeof(long long));
  const size_t vox = G > 0 ? (size_t)B * G * G * G : 0;
  if (G > 0) {
    a.vox_sum = reinterpret_cast<long long*>(ws + off); off += align256(vox * sizeof(long long));
    a.vox_cnt = reinterpret_cast<int*>(ws + off);       off += align256(vox * sizeof(int));
  }
  a.n_points_bits = 1;
  while (a.n_points_bits < 40 && (1ll << a.n_points_bits) <= N) ++a.n_points_bits;

  // the absmax word, the voxel sums and the voxel counts must start at zero
  if (G > 0) {
    const long long words = (long long)(off / 4);
    const int blocks = (int)((words + 256 * 8 - 1) / (256 * 8) < 65535 ? (words + 256 * 8 - 1) / (256 * 8) : 65535);
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(ws), words);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }

  int slice_cursor = 0;
  struct Chunk { MassTable tab; int n_obj; int obj_base; int max_slices; };
  // objects go to the device in tables of kMaxObjPerLaunch; grid mode needs every object's absmax
  // and bins finished before any voxel is read, so the passes run over all tables one after another
  const int n_chunks = (B + kMaxObjPerLaunch - 1) / kMaxObjPerLaunch;
  for (int pass = 0; pass < (G > 0 ? 4 : 2); ++pass) {
    slice_cursor = 0;
    for (int c = 0; c < n_chunks; ++c) {
      Chunk ch{};
      ch.obj_base = c * kMaxObjPerLaunch;
      ch.n_obj = B - ch.obj_base < kMaxObjPerLaunch ? B - ch.obj_base : kMaxObjPerLaunch;
      int max_pt_slices = 0;
      for (int t = 0; t < ch.n_obj; ++t) {
        const MassObj& o = objs[ch.obj_base + t];
        MassObjDev& d = ch.tab.o[t];
        d.pt_begin = o.pt_begin; d.n_pts = o.n_pts;
        d.lo[0] = o.lo[0]; d.lo[1] = o.lo[1]; d.lo[2] = o.lo[2]; d.h = o.h;
        const int pt_slices = (int)slices_points(o.n_pts);
        max_pt_slices = pt_slices > max_pt_slices ? pt_slices : max_pt_slices;
        d.n_slices = pt_slices;
        d.slice_begin = slice_cursor;
        slice_cursor += G > 0 ? (int)slices_voxels(G) : pt_slices;
      }
      a.obj_base = ch.obj_base;
      dim3 block(kMassBlock);
      if (G == 0) {
        if (pass == 0) {
          if (max_pt_slices > 0)
            hipLaunchKernelGGL(k_mass_points, dim3(max_pt_slices, ch.n_obj), block, 0, stream, a, ch.tab);
        } else {
          hipLaunchKernelGGL(k_mass_final, dim3(ch.n_obj), block, 0, stream, a, ch.tab, mass, n_used);
        }
      } else {
        if (pass == 0) {
          if (max_pt_slices > 0)
            hipLaunchKernelGGL(k_mass_absmax, dim3(max_pt_slices, ch.n_obj), block, 0, stream, a, ch.tab);
        } else if (pass == 1) {
          if (max_pt_slices > 0)
            hipLaunchKernelGGL(k_mass_bin, dim3(max_pt_slices, ch.n_obj), block, 0, stream, a, ch.tab);
        } else {
          for (int t = 0; t < ch.n_obj; ++t) ch.tab.o[t].n_slices = (int)slices_voxels(G);
          if (pass == 2)
            hipLaunchKernelGGL(k_mass_voxels, dim3((int)slices_voxels(G), ch.n_obj), block, 0, stream, a, ch.tab);
          else
            hipLaunchKernelGGL(k_mass_final, dim3(ch.n_obj), block, 0, stream, a, ch.tab, mass, n_used);
        }
      }
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

}  // namespace aura
