// Shared host/device helpers of libspt (gfx950 only, wave64).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/spt.h"

namespace spt {

constexpr int kWave = 64;
constexpr int kBlock = 256;  // 4 waves per workgroup everywhere

// ---- host side -----------------------------------------------------------

enum class Format { Invalid, Unsupported, CSR, COO2, DIA, ELL, COO3, CSF3, BCSR, DCSR, CSC };

// Validates the descriptor (Table 1 legality, pointers, sizes) and names the
// level composition. On Invalid/Unsupported the thread-local error is set.
Format recognize(const spt_tensor* T);

spt_status fail(spt_status code, const char* fmt, ...);
void clear_error();

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define SPT_CHECK_LAUNCH(what)                                                   \
  do {                                                                           \
    hipError_t e_ = hipGetLastError();                                           \
    if (e_ != hipSuccess)                                                        \
      return ::spt::fail(SPT_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e_)); \
  } while (0)

// Bump allocator over the caller's workspace.
struct Workspace {
  char* base;
  size_t size, used = 0;
  Workspace(void* p, size_t n) : base(static_cast<char*>(p)), size(n) {}
  template <typename T>
  T* take(size_t count) {
    size_t bytes = align_up(count * sizeof(T), 256);
    T* r = reinterpret_cast<T*>(base + used);
    used += bytes;
    return r;
  }
  bool ok() const { return used <= size; }
};

// ---- device side ---------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Workgroup barrier that orders LDS traffic only. __syncthreads() also waits for every
// outstanding global load of the wave (its fence covers global memory), which would
// serialise loads issued ahead for a later step; this one waits for the wave's LDS
// operations and then meets the other waves, so such loads stay in flight across it.
// Use it only where nothing written to global memory has to be seen by the workgroup.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its
// own L2. This maps blockIdx.x to a logical block id such that every XCD works
// on one contiguous range of logical blocks, so neighbouring blocks (which
// re-read each other's part of x) share an L2.
constexpr int kXcds = 8;
__device__ __forceinline__ int xcd_contiguous_block_id() {
  const int nb = gridDim.x, q = nb / kXcds, rem = nb % kXcds;
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  return xcd * q + (xcd < rem ? xcd : rem) + slot;
}

// First index in sorted a[0..n) whose value is >= target, found by the whole
// wave: every step probes 64 evenly spaced entries, so a 4M-entry array needs
// 4 dependent loads instead of 22. All lanes return the same result.
__device__ __forceinline__ int wave_lower_bound(const int32_t* __restrict__ a, int n,
                                                int target) {
  int lo = 0, hi = n;
  const int lane = lane_id();
  while (hi > lo) {
    int span = hi - lo;
    int step = (span + kWave - 1) / kWave;
    int idx = lo + lane * step;
    bool less = (idx < hi) && (a[idx] < target);
    int cnt = __popcll(__ballot(less));
    if (cnt == 0) {
      hi = lo;
    } else {
      int last_less = lo + (cnt - 1) * step;
      int nhi = last_less + step;
      hi = nhi < hi ? nhi : hi;
      lo = last_less + 1;
    }
  }
  return lo;
}

#endif  // __HIPCC__

}  // namespace spt
