// aura_voxel_downsample: Sec. 3.2.1 "Adaptive Sampling".
//
// The voxel size follows the object, s_voxel = cbrt(V_bound / N_target); the object's boundary box is cut into cubes
// of that side and every occupied cube is replaced by the mean position of its points.  The grid of an object is
// small (a few hundred to a few thousand cubes for N_target ~ 150), so it is held densely:
//   k_vox_zero    clears the cubes' sums and counts
//   k_vox_bin     one thread per point: cube index (fp32 decision chain), coordinates as 64-bit fixed point; spatially
//                 sorted points fall into the same cube in runs, a run is added up inside the wave and its last lane
//                 issues the atomics (integer sums: the result does not depend on the order in which they land)
//   k_vox_count   occupied cubes per block of 2048 cubes
//   k_vox_scan    exclusive scan of the block counts (one workgroup); object offsets
//   k_vox_emit    per block: position of every occupied cube in the output list, mean position, count
//   k_vox_point   per point: the list position of its cube
// Every object's cubes start at a multiple of 2048, so blocks never straddle objects.  All traffic is a few bytes per
// point plus the grid: the call is bound by launch latency.
#include "aura_device.hpp"
#include "launch.hpp"

namespace aura {

constexpr int kVoxBlock = 256;
constexpr int kVoxCellsPerThread = 8;
constexpr int kVoxCellsPerBlock = kVoxBlock * kVoxCellsPerThread;   // 2048

struct VoxCell {
  long long sum[3];   // fixed-point coordinate sums
  long long cnt;
};

struct VoxObjDev {
  long long pt_begin;
  int n_pts;
  float lo[3];
  float s;
  int dims[3];
  int cell_begin;     // first cube of the object in the concatenated grid (a multiple of 2048)
};

struct VoxTable {
  VoxObjDev o[kMaxObjPerLaunch];
};

struct VoxArgs {
  const float* xyz;
  VoxCell* cells;      // [total cells]
  int* cell_slot;      // [total cells]: list position of an occupied cube
  int* block_cnt;      // [blocks]
  int* block_off;      // [blocks + 1]
  int n_blocks;
  int shift;           // fixed-point scale 2^shift
  float* out_xyz;      // [capacity][3]
  int* out_count;      // [capacity] or nullptr
  long long capacity;
  int* out_offsets;    // [B + 1]
  int* voxel_of_point; // [N] or nullptr
  int n_obj;
};

__device__ __forceinline__ int vox_axis(float x, float lo, float s, int n) {
#pragma clang fp contract(off)
  const float t = x - lo;
  const float fl = floorf(t / s);
  return (fl >= (float)(n - 1)) ? n - 1 : ((fl > 0.0f) ? (int)fl : 0);
}

__device__ __forceinline__ int vox_cell(const VoxObjDev& ob, const float* __restrict__ p) {
  const int ix = vox_axis(p[0], ob.lo[0], ob.s, ob.dims[0]);
  const int iy = vox_axis(p[1], ob.lo[1], ob.s, ob.dims[1]);
  const int iz = vox_axis(p[2], ob.lo[2], ob.s, ob.dims[2]);
  return ob.cell_begin + (iz * ob.dims[1] + iy) * ob.dims[0] + ix;
}

__global__ __launch_bounds__(kVoxBlock) void k_vox_zero(VoxArgs a) {
  typedef uint32_t vox_u32x4 __attribute__((ext_vector_type(4)));
  vox_u32x4* __restrict__ z = reinterpret_cast<vox_u32x4*>(a.cells);
  const long long n = (long long)a.n_blocks * kVoxCellsPerBlock * (long long)(sizeof(VoxCell) / 16);
  for (long long i = (long long)blockIdx.x * kVoxBlock + threadIdx.x; i < n; i += (long long)gridDim.x * kVoxBlock)
    z[i] = vox_u32x4{0u, 0u, 0u, 0u};
}

__global__ __launch_bounds__(kVoxBlock) void k_vox_bin(VoxArgs a, VoxTable tab) {
  const VoxObjDev ob = tab.o[blockIdx.y];
  const int l0 = blockIdx.x * kVoxBlock;
  if (l0 >= ob.n_pts) return;                       // uniform: whole workgroups leave
  const int lane = threadIdx.x % kWave;
  const int li = l0 + threadIdx.x;
  const bool used = li < ob.n_pts;
  const long long i = ob.pt_begin + (used ? li : ob.n_pts - 1);
  const float* __restrict__ p = a.xyz + 3 * i;
  int cell = -1 - lane;                             // unused lanes: an id no neighbour shares
  long long q[3] = {0, 0, 0};
  if (used) {
    cell = vox_cell(ob, p);
#pragma unroll
    for (int c = 0; c < 3; ++c) q[c] = __double2ll_rn(ldexp((double)p[c], a.shift));
  }
  const int prev = __shfl_up(cell, 1, kWave), next = __shfl_down(cell, 1, kWave);
  const bool head = lane == 0 || prev != cell, tail = lane == kWave - 1 || next != cell;
  int start = head ? lane : 0;                      // lane of the run's first member
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) start = max(start, __shfl_up(start, o, kWave));
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      const long long up = __shfl_up(q[c], o, kWave);
      if (lane - o >= start) q[c] += up;
    }
  }
  if (used && tail) {
    VoxCell* cc = a.cells + cell;
#pragma unroll
    for (int c = 0; c < 3; ++c) atomicAdd(reinterpret_cast<unsigned long long*>(&cc->sum[c]), (unsigned long long)q[c]);
    atomicAdd(reinterpret_cast<unsigned long long*>(&cc->cnt), (unsigned long long)(lane - start + 1));
  }
}

// Number of occupied cubes among the thread's 8, and the workgroup's exclusive prefix of it.
__device__ __forceinline__ int vox_block_prefix(int mine, int* sh, int* total) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  int inc = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += up;
  }
  if (lane == kWave - 1) sh[wave] = inc;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kVoxBlock / kWave; ++w) {
    if (w < wave) before += sh[w];
    all += sh[w];
  }
  *total = all;
  return before + inc - mine;
}

__global__ __launch_bounds__(kVoxBlock) void k_vox_count(VoxArgs a) {
  __shared__ int sh[kVoxBlock / kWave];
  const long long c0 = (long long)blockIdx.x * kVoxCellsPerBlock + threadIdx.x * kVoxCellsPerThread;
  int mine = 0;
#pragma unroll
  for (int e = 0; e < kVoxCellsPerThread; ++e) mine += a.cells[c0 + e].cnt > 0 ? 1 : 0;
  int total;
  vox_block_prefix(mine, sh, &total);
  if (threadIdx.x == 0) a.block_cnt[blockIdx.x] = total;
}

// One workgroup: block_off = exclusive scan of block_cnt; out_offsets[b] = occupied cubes before object b.
__global__ __launch_bounds__(kVoxBlock) void k_vox_scan(VoxArgs a, VoxTable tab) {
  __shared__ int sh[kVoxBlock / kWave];
  __shared__ int s_carry;
  if (threadIdx.x == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < a.n_blocks; base += kVoxBlock) {
    const int j = base + threadIdx.x;
    const int mine = j < a.n_blocks ? a.block_cnt[j] : 0;
    int total;
    const int before = vox_block_prefix(mine, sh, &total);
    const int carry = s_carry;
    if (j < a.n_blocks) a.block_off[j] = carry + before;
    __syncthreads();                 // everyone has read the carry and the wave totals
    if (threadIdx.x == 0) s_carry = carry + total;
    __syncthreads();
  }
  if (threadIdx.x == 0) a.block_off[a.n_blocks] = s_carry;
  __syncthreads();
  for (int b = threadIdx.x; b <= a.n_obj; b += kVoxBlock)
    a.out_offsets[b] = b < a.n_obj ? a.block_off[tab.o[b].cell_begin / kVoxCellsPerBlock] : a.block_off[a.n_blocks];
}

__global__ __launch_bounds__(kVoxBlock) void k_vox_emit(VoxArgs a) {
  __shared__ int sh[kVoxBlock / kWave];
  const long long c0 = (long long)blockIdx.x * kVoxCellsPerBlock + threadIdx.x * kVoxCellsPerThread;
  long long cnt[kVoxCellsPerThread];
  int mine = 0;
#pragma unroll
  for (int e = 0; e < kVoxCellsPerThread; ++e) {
    cnt[e] = a.cells[c0 + e].cnt;
    mine += cnt[e] > 0 ? 1 : 0;
  }
  int total;
  long long slot = a.block_off[blockIdx.x] + vox_block_prefix(mine, sh, &total);
#pragma unroll
  for (int e = 0; e < kVoxCellsPerThread; ++e) {
    if (cnt[e] <= 0) {
      a.cell_slot[c0 + e] = -1;
      continue;
    }
    a.cell_slot[c0 + e] = (int)slot;
    if (slot < a.capacity) {
      const VoxCell cc = a.cells[c0 + e];
#pragma unroll
      for (int c = 0; c < 3; ++c) a.out_xyz[3 * slot + c] = (float)(ldexp((double)cc.sum[c], -a.shift) / (double)cc.cnt);
      if (a.out_count) a.out_count[slot] = (int)cc.cnt;
    }
    ++slot;
  }
}

__global__ __launch_bounds__(kVoxBlock) void k_vox_point(VoxArgs a, VoxTable tab) {
  const VoxObjDev ob = tab.o[blockIdx.y];
  const int li = blockIdx.x * kVoxBlock + threadIdx.x;
  if (li >= ob.n_pts) return;
  const long long i = ob.pt_begin + li;
  a.voxel_of_point[i] = a.cell_slot[vox_cell(ob, a.xyz + 3 * i)];
}

// ---------------------------------------------------------------- host side

static size_t vox_align256(size_t x) { return (x + 255) & ~(size_t)255; }

// s_voxel and the cubes per axis of one box; false when the box is not a box or the grid is out of range.
bool voxel_grid(const float* lo, const float* hi, int n_target, float* s_out, int* dims) {
  float e[3], emax = 0.0f;
  for (int a = 0; a < 3; ++a) {
    e[a] = hi[a] - lo[a];
    if (!(e[a] >= 0.0f) || e[a] > 3.0e38f) return false;
    emax = e[a] > emax ? e[a] : emax;
  }
  float s = (float)cbrt((double)e[0] * (double)e[1] * (double)e[2] / (double)n_target);
  if (!(s > 0.0f)) s = (float)((double)emax / cbrt((double)n_target));   // flat box: the longest side stands in
  if (!(s > 0.0f)) s = 1.0f;                                             // a single point
  *s_out = s;
  for (int a = 0; a < 3; ++a) {
    const float q = floorf(e[a] / s);
    if (!(q < (float)kVoxelMaxCells)) return false;
    dims[a] = (int)q + 1;
  }
  return (long long)dims[0] * dims[1] * dims[2] <= kVoxelMaxCells;
}

static long long vox_padded(long long cells) { return (cells + kVoxCellsPerBlock - 1) / kVoxCellsPerBlock * kVoxCellsPerBlock; }

long long voxel_padded_cells(long long cells) { return vox_padded(cells); }

size_t voxel_workspace_bytes(long long padded_cells) {
  const size_t blocks = (size_t)(padded_cells / kVoxCellsPerBlock);
  return vox_align256((size_t)padded_cells * sizeof(VoxCell)) + vox_align256((size_t)padded_cells * sizeof(int)) +
         vox_align256(blocks * sizeof(int)) + vox_align256((blocks + 1) * sizeof(int));
}

hipError_t launch_voxel_downsample(const float* xyz, const VoxObj* objs, int B, float max_abs, long long n_points,
                                   float* out_xyz, int* out_count, long long capacity, int* out_offsets,
                                   int* voxel_of_point, void* workspace, hipStream_t stream) {
  VoxTable tab{};
  long long cells = 0;
  int max_pts = 0;
  for (int b = 0; b < B; ++b) {
    VoxObjDev& d = tab.o[b];
    d.pt_begin = objs[b].pt_begin; d.n_pts = objs[b].n_pts; d.s = objs[b].s;
    for (int a = 0; a < 3; ++a) { d.lo[a] = objs[b].lo[a]; d.dims[a] = objs[b].dims[a]; }
    d.cell_begin = (int)cells;
    cells += vox_padded((long long)d.dims[0] * d.dims[1] * d.dims[2]);
    max_pts = d.n_pts > max_pts ? d.n_pts : max_pts;
  }
  VoxArgs a{};
  a.xyz = xyz;
  a.n_blocks = (int)(cells / kVoxCellsPerBlock);
  char* ws = static_cast<char*>(workspace);
  size_t off = 0;
  a.cells = reinterpret_cast<VoxCell*>(ws + off);   off += vox_align256((size_t)cells * sizeof(VoxCell));
  a.cell_slot = reinterpret_cast<int*>(ws + off);   off += vox_align256((size_t)cells * sizeof(int));
  a.block_cnt = reinterpret_cast<int*>(ws + off);   off += vox_align256((size_t)a.n_blocks * sizeof(int));
  a.block_off = reinterpret_cast<int*>(ws + off);
  // fixed point: |x| 2^shift n_points < 2^62 for every coordinate up to max_abs
  int e = 0, nbits = 1;
  frexpf(max_abs, &e);
  if (!(max_abs > 0.0f)) e = 0;
  while (nbits < 40 && (1ll << nbits) <= n_points) ++nbits;
  a.shift = 62 - e - nbits;
  a.out_xyz = out_xyz; a.out_count = out_count; a.capacity = capacity; a.out_offsets = out_offsets;
  a.voxel_of_point = voxel_of_point; a.n_obj = B;

  const dim3 block(kVoxBlock);
  const int zero_groups = a.n_blocks * 4 < 2048 ? a.n_blocks * 4 : 2048;
  hipLaunchKernelGGL(k_vox_zero, dim3(zero_groups), block, 0, stream, a);
  if (max_pts > 0) hipLaunchKernelGGL(k_vox_bin, dim3((max_pts + kVoxBlock - 1) / kVoxBlock, B), block, 0, stream, a, tab);
  hipLaunchKernelGGL(k_vox_count, dim3(a.n_blocks), block, 0, stream, a);
  hipLaunchKernelGGL(k_vox_scan, dim3(1), block, 0, stream, a, tab);
  hipLaunchKernelGGL(k_vox_emit, dim3(a.n_blocks), block, 0, stream, a);
  if (voxel_of_point && max_pts > 0)
    hipLaunchKernelGGL(k_vox_point, dim3((max_pts + kVoxBlock - 1) / kVoxBlock, B), block, 0, stream, a, tab);
  return hipGetLastError();
}

}  // namespace aura
