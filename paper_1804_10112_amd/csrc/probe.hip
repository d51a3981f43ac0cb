// Measurement aids: the pure streaming read and the pure random gather that
// bound the sparse kernels, as stand-alone kernels (no counterpart in the paper).
#include "common.hpp"

namespace spt {

template <typename V>
__global__ __launch_bounds__(kBlock) void probe_read_kernel(const V* __restrict__ a, size_t n,
                                                            float* __restrict__ sink) {
  constexpr int IPT = 4;
  const size_t base = (size_t)blockIdx.x * kBlock * IPT + threadIdx.x;
  V v[IPT];
#pragma unroll
  for (int k = 0; k < IPT; ++k) {
    const size_t i = base + (size_t)k * kBlock;
    v[k] = i < n ? __builtin_nontemporal_load(a + i) : V(0);
  }
  float s = 0;
#pragma unroll
  for (int k = 0; k < IPT; ++k) s += reinterpret_cast<const float*>(&v[k])[0];
  if (s == 12345.678f) sink[0] = s;  // keeps the loads alive, practically never true
}

template <typename T>
__global__ __launch_bounds__(kBlock) void probe_gather_kernel(const int32_t* __restrict__ idx,
                                                              int64_t n, const T* __restrict__ table,
                                                              T* __restrict__ out) {
  // four independent gathers per lane, all issued before the first store: a kernel that keeps
  // several gathers in flight per lane must not be able to outrun its own yardstick
  constexpr int IPT = 4;
  const int64_t base = (int64_t)blockIdx.x * kBlock * IPT + threadIdx.x;
  int32_t j[IPT];
  T v[IPT];
#pragma unroll
  for (int k = 0; k < IPT; ++k) {
    const int64_t p = base + (int64_t)k * kBlock;
    j[k] = p < n ? __builtin_nontemporal_load(idx + p) : 0;
  }
#pragma unroll
  for (int k = 0; k < IPT; ++k) v[k] = table[j[k]];
#pragma unroll
  for (int k = 0; k < IPT; ++k) {
    const int64_t p = base + (int64_t)k * kBlock;
    if (p < n) __builtin_nontemporal_store(v[k], out + p);
  }
}

}  // namespace spt

using namespace spt;

extern "C" spt_status spt_probe_read(const void* src, size_t bytes, int32_t lane_bytes, void* sink,
                                     void* stream) {
  clear_error();
  if (!src || !sink || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15))
    return fail(SPT_ERR_INVALID_ARG, "probe_read: null or unaligned arguments");
  hipStream_t s = static_cast<hipStream_t>(stream);
  typedef float f4 __attribute__((ext_vector_type(4)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  const size_t n = bytes / lane_bytes;
  const unsigned grid = (unsigned)((n + kBlock * 4 - 1) / (kBlock * 4));
  if (grid == 0) return SPT_OK;
  if (lane_bytes == 16)
    hipLaunchKernelGGL(probe_read_kernel<f4>, dim3(grid), dim3(kBlock), 0, s,
                       static_cast<const f4*>(src), n, static_cast<float*>(sink));
  else if (lane_bytes == 8)
    hipLaunchKernelGGL(probe_read_kernel<f2>, dim3(grid), dim3(kBlock), 0, s,
                       static_cast<const f2*>(src), n, static_cast<float*>(sink));
  else if (lane_bytes == 4)
    hipLaunchKernelGGL(probe_read_kernel<float>, dim3(grid), dim3(kBlock), 0, s,
                       static_cast<const float*>(src), n, static_cast<float*>(sink));
  else
    return fail(SPT_ERR_INVALID_ARG, "probe_read: lane_bytes must be 4, 8 or 16");
  SPT_CHECK_LAUNCH("probe_read");
  return SPT_OK;
}

extern "C" spt_status spt_probe_gather(const int32_t* idx, int64_t n, const void* table,
                                       int32_t dtype, void* out, void* stream) {
  clear_error();
  if (!idx || !table || !out || n < 0)
    return fail(SPT_ERR_INVALID_ARG, "probe_gather: null argument or negative count");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = (unsigned)((n + 4 * kBlock - 1) / (4 * kBlock));
  if (grid == 0) return SPT_OK;
  if (dtype == SPT_F64)
    hipLaunchKernelGGL(probe_gather_kernel<double>, dim3(grid), dim3(kBlock), 0, s, idx, n,
                       static_cast<const double*>(table), static_cast<double*>(out));
  else if (dtype == SPT_F32)
    hipLaunchKernelGGL(probe_gather_kernel<float>, dim3(grid), dim3(kBlock), 0, s, idx, n,
                       static_cast<const float*>(table), static_cast<float*>(out));
  else
    return fail(SPT_ERR_INVALID_ARG, "probe_gather: unknown dtype %d", dtype);
  SPT_CHECK_LAUNCH("probe_gather");
  return SPT_OK;
}
