// Pieces of the radix machinery shared by the COO->CSR sort and the binned
// COO SpMV: digit extraction and the per-tile digit histogram.
#pragma once
#include "common.hpp"

namespace spt {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortIPT = 16;
constexpr int kSortTile = kSortIPT * kBlock;  // 4096 records per workgroup
constexpr int kWaves = kBlock / kWave;

inline int bits_for(int64_t dim) {
  int b = 1;
  while (b < 31 && ((int64_t)1 << b) < dim) ++b;
  return b;
}

__device__ __forceinline__ int digit_of(int32_t key, int shift) {
  return ((uint32_t)key >> shift) & (kRadix - 1);
}

// One more key with digit d in each of the wave's 64 lanes (all active, lane order =
// key order up to a fixed stride). Sorted input (a long row, a long fibre) gives
// neighbouring lanes the same digit, and separate LDS atomics on one counter are
// serialised: the first lane of every run of equal digits adds the run's length.
__device__ __forceinline__ void count_digit_runs(int* cnt, int d) {
  const int lane = lane_id();
  // lane l receives lane l-1's digit through the data-parallel-primitive path
  // (wave_shr:1; lane 0 keeps its own), not through the LDS crossbar
  const int prev = __builtin_amdgcn_update_dpp(d, d, 0x138, 0xf, 0xf, false);
  const bool head = lane == 0 || d != prev;
  const uint64_t heads = __ballot(head);
  if (head) {
    const uint64_t above = lane == kWave - 1 ? 0 : heads >> (lane + 1);
    const int len = above ? __ffsll(static_cast<long long>(above)) : kWave - lane;
    atomicAdd(&cnt[d], len);
  }
}

// hist[d * ntiles + tile] = number of keys of this tile whose digit is d.
// A workgroup counts kHistGroup consecutive tiles, each wave a tile at a time into
// that tile's own LDS counters, and thread d then stores digit d's counts of all
// its tiles side by side: the layout is digit-major for the scan that follows, and
// one count per tile and digit stored on its own would be a scattered 4-byte write.
// VEC: 16-byte key loads (needs a 16-byte aligned key array).
constexpr int kHistGroup = 8;
template <bool VEC>
__global__ __launch_bounds__(kBlock) void radix_hist_kernel(const int32_t* __restrict__ key, int n,
                                                            int shift, int ntiles,
                                                            int32_t* __restrict__ hist) {
  __shared__ int s_cnt[kHistGroup][kRadix];
  for (int q = threadIdx.x; q < kHistGroup * kRadix; q += kBlock) (&s_cnt[0][0])[q] = 0;
  __syncthreads();
  const int tile0 = xcd_contiguous_block_id() * kHistGroup;  // neighbours store into the same cache lines
  const int lane = lane_id();
  for (int t = wave_id(); t < kHistGroup && tile0 + t < ntiles; t += kWaves) {
    const int base = (tile0 + t) * kSortTile;
    int* cnt = s_cnt[t];
    if (VEC) {
      typedef int32_t i4 __attribute__((ext_vector_type(4)));
#pragma unroll 8
      for (int q = 0; q < kSortTile / (4 * kWave); ++q) {
        const int i = base + (q * kWave + lane) * 4;
        if (base + (q + 1) * kWave * 4 <= n) {  // the whole wave is inside the array
          const i4 k4 = __builtin_nontemporal_load(reinterpret_cast<const i4*>(key + i));
#pragma unroll
          for (int r = 0; r < 4; ++r) count_digit_runs(cnt, digit_of(k4[r], shift));
        } else if (i + 4 <= n) {
          const i4 k4 = __builtin_nontemporal_load(reinterpret_cast<const i4*>(key + i));
#pragma unroll
          for (int r = 0; r < 4; ++r) atomicAdd(&cnt[digit_of(k4[r], shift)], 1);
        } else {
          for (int r = 0; r < 4; ++r)
            if (i + r < n) atomicAdd(&cnt[digit_of(key[i + r], shift)], 1);
        }
      }
    } else {
#pragma unroll 4
      for (int q = 0; q < kSortTile / kWave; ++q) {
        const int i = base + q * kWave + lane;
        if (i < n) atomicAdd(&cnt[digit_of(key[i], shift)], 1);
      }
    }
  }
  __syncthreads();
  const int nt = min(kHistGroup, ntiles - tile0);
  int32_t* out = hist + (int64_t)threadIdx.x * ntiles + tile0;
  for (int t = 0; t < nt; ++t) out[t] = s_cnt[t][threadIdx.x];
}


#if defined(__HIPCC__)
// Enqueues the histogram of digit (key >> shift) & 255 for every tile of kSortTile keys.
inline spt_status launch_radix_hist(const int32_t* key, int n, int shift, int ntiles, int32_t* hist,
                                    hipStream_t s) {
  if ((reinterpret_cast<uintptr_t>(key) & 15) == 0)
    hipLaunchKernelGGL(radix_hist_kernel<true>, dim3((ntiles + kHistGroup - 1) / kHistGroup),
                       dim3(kBlock), 0, s, key, n, shift, ntiles, hist);
  else
    hipLaunchKernelGGL(radix_hist_kernel<false>, dim3((ntiles + kHistGroup - 1) / kHistGroup),
                       dim3(kBlock), 0, s, key, n, shift, ntiles, hist);
  SPT_CHECK_LAUNCH("radix_hist");
  return SPT_OK;
}
#endif

}  // namespace spt
