// Device-wide prefix sum of int32 (two or three plain kernels, no spin waits):
// per-tile sums -> (beyond 2048 tiles: one workgroup scans the tile sums) -> per-tile scan + offset.
// This is the GPU form of Table 3's append_finalize (pos = running sum of the
// per-parent counts) and of the digit offsets of every radix-sort pass.
#pragma once
#include "common.hpp"

namespace spt {

constexpr int kScanIPT = 16;
constexpr int kScanTile = kScanIPT * kBlock;
constexpr int64_t kScanSelfTiles = 2048;  // up to here a workgroup re-adds the earlier tiles' sums (8 KB)

inline int64_t scan_tiles(int64_t n) { return (n + kScanTile - 1) / kScanTile; }
inline size_t scan_workspace(int64_t n) { return align_up((size_t)(scan_tiles(n) + 1) * 4, 256); }

#if defined(__HIPCC__)

// Inclusive sum over the workgroup of one int per thread; returns the inclusive
// value, *total receives the workgroup sum. One __syncthreads inside plus one
// at entry (protects the shared array between consecutive calls).
__device__ __forceinline__ int block_inclusive_sum(int v, int* total) {
  __shared__ int s_w[kBlock / kWave];
  const int lane = lane_id(), w = wave_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int u = __shfl_up(v, d);
    if (lane >= d) v += u;
  }
  __syncthreads();
  if (lane == kWave - 1) s_w[w] = v;
  __syncthreads();
  int pre = 0, tot = 0;
#pragma unroll
  for (int u = 0; u < kBlock / kWave; ++u) {
    if (u < w) pre += s_w[u];
    tot += s_w[u];
  }
  *total = tot;
  return v + pre;
}

static __global__ __launch_bounds__(kBlock) void scan_tile_sums_kernel(const int32_t* __restrict__ in,
                                                                int64_t n,
                                                                int32_t* __restrict__ tile_sum) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile;
  int s = 0;
#pragma unroll
  for (int k = 0; k < kScanIPT; ++k) {
    int64_t i = base + k * kBlock + threadIdx.x;
    if (i < n) s += in[i];
  }
  int total;
  block_inclusive_sum(s, &total);
  if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// Single workgroup: exclusive scan of tile_sum[0..ntiles) in place.
static __global__ __launch_bounds__(kBlock) void scan_spine_kernel(int32_t* __restrict__ tile_sum,
                                                            int64_t ntiles) {
  int carry = 0;
  for (int64_t b = 0; b < ntiles; b += kBlock) {
    int64_t i = b + threadIdx.x;
    int v = i < ntiles ? tile_sum[i] : 0;
    int total;
    int incl = block_inclusive_sum(v, &total);
    if (i < ntiles) tile_sum[i] = carry + incl - v;
    carry += total;
  }
}

// out[i] = sum of in[0..i) (+ in[i] if INCLUSIVE). in may equal out.
// SELF: tile_off holds the tile sums themselves and every workgroup adds up the sums of the
// tiles before its own (a few KB from L2), which saves the launch of the spine kernel.
template <bool INCLUSIVE, bool SELF = false>
__global__ __launch_bounds__(kBlock) void scan_apply_kernel(const int32_t* in, int64_t n,
                                                            const int32_t* __restrict__ tile_off,
                                                            int32_t* out) {
  typedef int32_t i4 __attribute__((ext_vector_type(4)));
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanIPT;
  // a thread's 16 consecutive values move as four 16-byte words when they are all inside
  // the array and both arrays are 16-byte aligned there (single 4-byte stores at a 64-byte
  // lane stride cost a memory transaction each)
  const bool wide = base + kScanIPT <= n &&
                    ((reinterpret_cast<uintptr_t>(in + base) | reinterpret_cast<uintptr_t>(out + base)) & 15) == 0;
  int v[kScanIPT];
  int s = 0;
  if (wide) {
#pragma unroll
    for (int q = 0; q < kScanIPT / 4; ++q) {
      const i4 w = *reinterpret_cast<const i4*>(in + base + 4 * q);
#pragma unroll
      for (int r = 0; r < 4; ++r) v[4 * q + r] = w[r];
    }
  } else {
#pragma unroll
    for (int k = 0; k < kScanIPT; ++k) v[k] = (base + k < n) ? in[base + k] : 0;
  }
#pragma unroll
  for (int k = 0; k < kScanIPT; ++k) s += v[k];
  int before = 0;  // sum of everything in the tiles before this one
  if (SELF) {
    int part = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kBlock) part += tile_off[t];
    block_inclusive_sum(part, &before);
  } else {
    before = tile_off[blockIdx.x];
  }
  int total;
  int run = block_inclusive_sum(s, &total) - s + before;
#pragma unroll
  for (int k = 0; k < kScanIPT; ++k) {
    const int x = v[k];
    v[k] = INCLUSIVE ? run + x : run;
    run += x;
  }
  if (wide) {
#pragma unroll
    for (int q = 0; q < kScanIPT / 4; ++q) {
      i4 w;
#pragma unroll
      for (int r = 0; r < 4; ++r) w[r] = v[4 * q + r];
      *reinterpret_cast<i4*>(out + base + 4 * q) = w;
    }
  } else {
#pragma unroll
    for (int k = 0; k < kScanIPT; ++k)
      if (base + k < n) out[base + k] = v[k];
  }
}

// Enqueues the kernels. tmp needs scan_workspace(n) bytes.
template <bool INCLUSIVE>
inline spt_status device_scan_i32(const int32_t* in, int32_t* out, int64_t n, int32_t* tmp,
                                  hipStream_t s) {
  if (n <= 0) return SPT_OK;
  const int64_t nt = scan_tiles(n);
  hipLaunchKernelGGL(scan_tile_sums_kernel, dim3((unsigned)nt), dim3(kBlock), 0, s, in, n, tmp);
  SPT_CHECK_LAUNCH("scan_tile_sums");
  if (nt <= kScanSelfTiles) {  // two kernels: the apply kernel sums the earlier tiles' sums itself
    hipLaunchKernelGGL((scan_apply_kernel<INCLUSIVE, true>), dim3((unsigned)nt), dim3(kBlock), 0, s, in, n,
                       tmp, out);
    SPT_CHECK_LAUNCH("scan_apply");
    return SPT_OK;
  }
  hipLaunchKernelGGL(scan_spine_kernel, dim3(1), dim3(kBlock), 0, s, tmp, nt);
  SPT_CHECK_LAUNCH("scan_spine");
  hipLaunchKernelGGL((scan_apply_kernel<INCLUSIVE, false>), dim3((unsigned)nt), dim3(kBlock), 0, s, in, n,
                     tmp, out);
  SPT_CHECK_LAUNCH("scan_apply");
  return SPT_OK;
}

#endif  // __HIPCC__
}  // namespace spt
