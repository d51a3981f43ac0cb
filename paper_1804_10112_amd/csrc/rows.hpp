// pos of a compressed level from the ordered coordinates of its parent level, shared by
// the COO -> CSR conversion and the packers.
#pragma once
#include "common.hpp"

namespace spt {

// pos of the compressed column level from the sorted rows. Table 3 assembles pos as
// per-parent counts (append_edges) followed by a running sum (append_finalize); on sorted
// rows that running sum is known directly: pos[r] = position of the first entry whose row
// is >= r. The thread of entry p, whose predecessor lies in row a and which lies in row b,
// therefore stores p into pos[a+1 .. b] (nothing if a == b), and the last entry's thread
// stores n into the rest: every element of pos is written exactly once, without atomics
// or a scan. Ranges longer than 16 rows (runs of empty rows) are written by the whole wave.
static __device__ __forceinline__ void store_pos_range(int32_t* __restrict__ pos, int lo, int hi, int val) {
  const bool big = hi - lo > 16;
  if (!big)
    for (int r = lo + 1; r <= hi; ++r) pos[r] = val;
  uint64_t todo = __ballot(big);
  while (todo) {
    const int src = __ffsll(static_cast<long long>(todo)) - 1;
    todo &= todo - 1;
    const int l = __shfl(lo, src), h = __shfl(hi, src), v = __shfl(val, src);
    for (int r = l + 1 + lane_id(); r <= h; r += kWave) pos[r] = v;
  }
}
template <bool VEC>
// n_dev: if not null, the number of entries is read from there (a count that an earlier
// kernel produced); the grid then covers the capacity n and the lanes beyond the count idle.
static __global__ __launch_bounds__(kBlock) void pos_from_sorted_rows_kernel(const int32_t* __restrict__ row,
                                                                      int n, int nrows,
                                                                      int32_t* __restrict__ pos,
                                                                      const int64_t* __restrict__ n_dev) {
  typedef int32_t i4 __attribute__((ext_vector_type(4)));
  if (n_dev) n = static_cast<int>(*n_dev);
  const int p0 = (blockIdx.x * kBlock + threadIdx.x) * 4;  // four consecutive entries per lane
  int r4[4];
  if (VEC && p0 + 4 <= n) {
    const i4 v = __builtin_nontemporal_load(reinterpret_cast<const i4*>(row + p0));
#pragma unroll
    for (int k = 0; k < 4; ++k) r4[k] = v[k];
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) r4[k] = p0 + k < n ? row[p0 + k] : 0;
  }
  int a = (p0 > 0 && p0 < n) ? row[p0 - 1] : -1;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const bool live = p0 + k < n;  // every lane of a wave takes part in the long ranges
    store_pos_range(pos, live ? a : 0, live ? r4[k] : 0, p0 + k);
    const bool last = live && p0 + k == n - 1;
    if (__any(last)) store_pos_range(pos, last ? r4[k] : 0, last ? nrows : 0, n);
    a = r4[k];
  }
}

// Enqueues pos_from_sorted_rows_kernel for n > 0 ordered row coordinates (with n_dev: for at
// most n of them, the count being in device memory; a count of 0 leaves pos untouched).
inline spt_status launch_pos_from_sorted_rows(const int32_t* rows, int n, int nrows, int32_t* pos,
                                              hipStream_t s, const int64_t* n_dev = nullptr) {
  const unsigned grid = (unsigned)((n + 4 * kBlock - 1) / (4 * kBlock));
  if ((reinterpret_cast<uintptr_t>(rows) & 15) == 0)
    hipLaunchKernelGGL(pos_from_sorted_rows_kernel<true>, dim3(grid), dim3(kBlock), 0, s, rows, n,
                       nrows, pos, n_dev);
  else
    hipLaunchKernelGGL(pos_from_sorted_rows_kernel<false>, dim3(grid), dim3(kBlock), 0, s, rows, n,
                       nrows, pos, n_dev);
  SPT_CHECK_LAUNCH("pos_from_sorted_rows");
  return SPT_OK;
}

}  // namespace spt
