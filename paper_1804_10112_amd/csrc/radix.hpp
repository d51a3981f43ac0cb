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

// hist[d * ntiles + tile] = number of keys of this tile whose digit is d.
// VEC: 16-byte key loads (needs a 16-byte aligned key array).
template <bool VEC>
__global__ __launch_bounds__(kBlock) void radix_hist_kernel(const int32_t* __restrict__ key, int n,
                                                            int shift, int ntiles,
                                                            int32_t* __restrict__ hist) {
  __shared__ int s_cnt[kWaves][kRadix];
  for (int q = threadIdx.x; q < kWaves * kRadix; q += kBlock) (&s_cnt[0][0])[q] = 0;
  __syncthreads();
  const int base = blockIdx.x * kSortTile;
  int* cnt = s_cnt[wave_id()];
  if (VEC) {
    typedef int32_t i4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int q = 0; q < kSortIPT / 4; ++q) {
      const int i = base + (q * kBlock + threadIdx.x) * 4;
      if (i + 4 <= n) {
        const i4 k4 = __builtin_nontemporal_load(reinterpret_cast<const i4*>(key + i));
#pragma unroll
        for (int r = 0; r < 4; ++r) atomicAdd(&cnt[digit_of(k4[r], shift)], 1);
      } else {
        for (int r = 0; r < 4; ++r)
          if (i + r < n) atomicAdd(&cnt[digit_of(key[i + r], shift)], 1);
      }
    }
  } else {
#pragma unroll
    for (int k = 0; k < kSortIPT; ++k) {
      const int i = base + k * kBlock + threadIdx.x;
      if (i < n) atomicAdd(&cnt[digit_of(key[i], shift)], 1);
    }
  }
  __syncthreads();
  int tot = 0;
#pragma unroll
  for (int u = 0; u < kWaves; ++u) tot += s_cnt[u][threadIdx.x];
  hist[(int64_t)threadIdx.x * ntiles + blockIdx.x] = tot;
}


#if defined(__HIPCC__)
// Enqueues the histogram of digit (key >> shift) & 255 for every tile of kSortTile keys.
inline spt_status launch_radix_hist(const int32_t* key, int n, int shift, int ntiles, int32_t* hist,
                                    hipStream_t s) {
  if ((reinterpret_cast<uintptr_t>(key) & 15) == 0)
    hipLaunchKernelGGL(radix_hist_kernel<true>, dim3(ntiles), dim3(kBlock), 0, s, key, n, shift,
                       ntiles, hist);
  else
    hipLaunchKernelGGL(radix_hist_kernel<false>, dim3(ntiles), dim3(kBlock), 0, s, key, n, shift,
                       ntiles, hist);
  SPT_CHECK_LAUNCH("radix_hist");
  return SPT_OK;
}
#endif

}  // namespace spt
