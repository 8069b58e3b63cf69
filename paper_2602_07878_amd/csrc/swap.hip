// KV-block gather/scatter of the preemption swap path (arXiv 2602.07878,
// Sec. 5.1.2 "Swapping") and two plain streaming probes, for gfx950.
//
// No arithmetic: every lane moves 16 bytes per access.  The work list is the
// set of (plane, pair) chunks in plane-major order.  Each wavefront copies
// whole chunks by itself, 16 KiB at a time (16 loads of 16 bytes per lane in
// flight, then 16 stores), the four wavefronts of a workgroup take adjacent
// chunks and switch between reading and writing together, and the grid covers
// three quarters of the CUs only.  All of that is measured DRAM behaviour of
// a copy on this part: long same-direction bursts from few requesters lose the
// least to read/write turnaround (5.2 -> 6.2 TB/s of traffic on the gather of
// the 64-victim configuration compared with one workgroup per chunk on every CU).

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 256;
constexpr int kUnroll = 8;  // 16-byte accesses in flight per lane

__device__ __forceinline__ u32x4 ld_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_stream(u32x4* p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// Copy `n16` 16-byte units from s to d with the whole workgroup.
__device__ __forceinline__ void wg_copy(const u32x4* __restrict__ s, u32x4* __restrict__ d,
                                        int64_t n16) {
  int64_t i = threadIdx.x;
  for (; i + (kUnroll - 1) * kCopyThreads < n16; i += kUnroll * kCopyThreads) {
    u32x4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) r[u] = ld_stream(s + i + u * kCopyThreads);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) st_stream(d + i + u * kCopyThreads, r[u]);
  }
  for (; i < n16; i += kCopyThreads) st_stream(d + i, ld_stream(s + i));
}

constexpr int kBurst = 16;                       // 16-byte accesses per lane per phase
constexpr int kCopyWaves = kCopyThreads / kWaveSize;

__global__ __launch_bounds__(kCopyThreads) void swap_blocks(const SwapParams p) {
  const int64_t nchunks = (int64_t)p.num_planes * p.n_pairs;
  const int64_t n16 = p.block_bytes / 16;
  const int lane = threadIdx.x & (kWaveSize - 1);
  const int64_t wid = (int64_t)blockIdx.x * kCopyWaves + threadIdx.x / kWaveSize;
  const int64_t nw = (int64_t)gridDim.x * kCopyWaves;
  // every wavefront runs the same number of rounds: the barriers below are workgroup-wide
  const int64_t iters = (nchunks + nw - 1) / nw;
  for (int64_t it = 0; it < iters; ++it) {
    const int64_t c = wid + it * nw;
    const bool live = c < nchunks;
    const int64_t cc = live ? c : nchunks - 1;
    // plane-major order: consecutive chunks are consecutive pairs of one plane
    const int plane = (int)(cc / p.n_pairs);
    const int pair = (int)(cc % p.n_pairs);
    const int64_t sb = p.src_slot_is_pair ? pair : __builtin_amdgcn_readfirstlane(p.mapping[2 * pair]);
    const int64_t db = p.dst_slot_is_pair ? pair : __builtin_amdgcn_readfirstlane(p.mapping[2 * pair + 1]);
    const u32x4* s = reinterpret_cast<const u32x4*>(p.src + plane * p.src_plane_stride +
                                                    sb * p.block_bytes);
    u32x4* d = reinterpret_cast<u32x4*>(p.dst + plane * p.dst_plane_stride + db * p.block_bytes);
    for (int64_t base = 0; base < n16; base += kBurst * kWaveSize) {
      u32x4 r[kBurst];
      const bool full = base + kBurst * kWaveSize <= n16;   // wave-uniform
      const u32x4* sp = s + base + lane;
      u32x4* dp = d + base + lane;
      if (live) {
        if (full) {
#pragma unroll
          for (int u = 0; u < kBurst; ++u) r[u] = ld_stream(sp + u * kWaveSize);
        } else {
#pragma unroll
          for (int u = 0; u < kBurst; ++u)
            if (base + u * kWaveSize + lane < n16) r[u] = ld_stream(sp + u * kWaveSize);
        }
      }
      __syncthreads();   // the workgroup reads together, then writes together
      if (live) {
        if (full) {
#pragma unroll
          for (int u = 0; u < kBurst; ++u) st_stream(dp + u * kWaveSize, r[u]);
        } else {
#pragma unroll
          for (int u = 0; u < kBurst; ++u)
            if (base + u * kWaveSize + lane < n16) st_stream(dp + u * kWaveSize, r[u]);
        }
      }
    }
  }
}

__global__ __launch_bounds__(kCopyThreads) void probe_copy(const u32x4* __restrict__ s,
                                                           u32x4* __restrict__ d, int64_t n16) {
  constexpr int64_t span = (int64_t)kUnroll * kCopyThreads;  // units per workgroup step
  for (int64_t base = (int64_t)blockIdx.x * span; base < n16; base += (int64_t)gridDim.x * span) {
    const int64_t left = n16 - base;
    wg_copy(s + base, d + base, left < span ? left : span);
  }
}

__global__ __launch_bounds__(kCopyThreads) void probe_read(const u32x4* __restrict__ s,
                                                           u32x4* __restrict__ sink, int64_t n16) {
  constexpr int64_t span = (int64_t)kUnroll * kCopyThreads;
  u32x4 acc = {0, 0, 0, 0};
  for (int64_t base = (int64_t)blockIdx.x * span; base < n16; base += (int64_t)gridDim.x * span) {
    u32x4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t i = base + threadIdx.x + u * kCopyThreads;
      r[u] = i < n16 ? ld_stream(s + i) : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= r[u];
  }
  // fold the workgroup's checksum into one 16-byte value (keeps the loads live)
  __shared__ u32x4 red[kCopyThreads];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int off = kCopyThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] ^= red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) sink[blockIdx.x] = red[0];
}

int grid_for_device(int wgs_per_cu) {
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) == hipSuccess) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cus = v;
  }
  return cus * wgs_per_cu;
}

}  // namespace

hipError_t launch_swap(const SwapParams& p, hipStream_t s, int max_workgroups) {
  const int64_t nchunks = (int64_t)p.num_planes * p.n_pairs;
  int64_t grid = grid_for_device(3) / 4;   // three workgroups per four CUs
  if (max_workgroups > 0 && grid > max_workgroups) grid = max_workgroups;
  const int64_t need = (nchunks + kCopyWaves - 1) / kCopyWaves;
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(swap_blocks, dim3((unsigned)grid), dim3(kCopyThreads), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
  const int64_t n16 = (int64_t)(bytes / 16);
  int64_t grid = grid_for_device(8);
  const int64_t need = (n16 + kUnroll * kCopyThreads - 1) / (kUnroll * kCopyThreads);
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(probe_copy, dim3((unsigned)grid), dim3(kCopyThreads), 0, s,
                     reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), n16);
  return hipGetLastError();
}

hipError_t launch_probe_read(const void* src, void* sink, size_t bytes, hipStream_t s) {
  const int64_t n16 = (int64_t)(bytes / 16);
  int64_t grid = grid_for_device(8);
  if (grid > 4096) grid = 4096;  // sink holds 64 KiB = 4096 checksums
  const int64_t need = (n16 + kUnroll * kCopyThreads - 1) / (kUnroll * kCopyThreads);
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(probe_read, dim3((unsigned)grid), dim3(kCopyThreads), 0, s,
                     reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(sink), n16);
  return hipGetLastError();
}

}  // namespace pkv
