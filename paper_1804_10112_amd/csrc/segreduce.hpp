// Workgroup-level segmented reduction building blocks (wave64, 256 threads).
//
// The paper removes duplicates of an ordered, non-unique level with a
// deduplication loop that scans ahead over equal coordinates (Section 4.3).
// On the GPU the same aggregation is a segmented reduction: every position
// whose coordinate differs from its predecessor is a segment head, and each
// segment's sum is produced without atomics. A workgroup owns a fixed chunk of
// consecutive positions; the part of the chunk that continues a segment begun
// in an earlier chunk leaves the workgroup as one (key, partial) carry.
#pragma once
#include "common.hpp"

namespace spt {

// Per-thread summary of its consecutive items: f = a head occurs among them,
// v = sum after the last head (or of everything if f == 0), k = key of the
// last head (or -1). Summaries combine associatively, earlier operand first.
template <typename A>
struct SegSum {
  int f;
  A v;
  int k;
};

template <typename A>
__device__ __forceinline__ SegSum<A> seg_combine(const SegSum<A>& a, const SegSum<A>& b) {
  SegSum<A> r;
  r.f = a.f | b.f;
  r.v = b.f ? b.v : a.v + b.v;
  r.k = b.f ? b.k : a.k;
  return r;
}

template <typename A>
struct SegScanStorage {
  int f[kBlock / kWave];
  A v[kBlock / kWave];
  int k[kBlock / kWave];
};

// Exclusive segmented scan over the 256 threads of the workgroup, in thread
// order. Thread 0 receives the identity (f=0, v=0, k=-1).
// Contains one __syncthreads(); all threads must call it.
template <typename A>
__device__ __forceinline__ SegSum<A> block_seg_exclusive_scan(SegSum<A> me,
                                                              SegScanStorage<A>& st) {
  const int lane = lane_id(), w = wave_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    SegSum<A> up;
    up.f = __shfl_up(me.f, d);
    up.v = __shfl_up(me.v, d);
    up.k = __shfl_up(me.k, d);
    if (lane >= d) me = seg_combine(up, me);
  }
  if (lane == kWave - 1) {
    st.f[w] = me.f;
    st.v[w] = me.v;
    st.k[w] = me.k;
  }
  __syncthreads();
  SegSum<A> pre{0, A(0), -1};
  for (int u = 0; u < w; ++u) pre = seg_combine(pre, SegSum<A>{st.f[u], st.v[u], st.k[u]});
  SegSum<A> incl = seg_combine(pre, me);
  SegSum<A> ex;
  ex.f = __shfl_up(incl.f, 1);
  ex.v = __shfl_up(incl.v, 1);
  ex.k = __shfl_up(incl.k, 1);
  if (lane == 0) ex = pre;
  return ex;
}

// Adds the carries to y. Carries of one row are consecutive; the thread at the
// start of a run adds the whole run in order (deterministic). The sum of a run
// is formed in double also for float data.
// A choice between two kernels made on the device: an earlier kernel writes kSelectFlags flags,
// both candidates are launched, and each runs only if "any flag set" equals its `want`.
constexpr int kSelectFlags = 64;  // one per lane of a wave
__device__ __forceinline__ bool selected(const int32_t* __restrict__ select, int want) {
  if (!select) return true;
  const int any = __ballot(select[threadIdx.x & (kSelectFlags - 1)] != 0) != 0;
  return any == want;
}

template <typename T>
__global__ __launch_bounds__(kBlock) void carry_fixup_kernel(int n,
                                                             const int32_t* __restrict__ carry_key,
                                                             const T* __restrict__ carry_val,
                                                             T* __restrict__ y,
                                                             const int32_t* __restrict__ select = nullptr,
                                                             int want = 0) {
  if (!selected(select, want)) return;
  const int w = blockIdx.x * kBlock + threadIdx.x;
  if (w >= n) return;
  const int32_t key = carry_key[w];
  if (key < 0) return;
  if (w > 0 && carry_key[w - 1] == key) return;
  double s = 0;
  for (int u = w; u < n && carry_key[u] == key; ++u) s += (double)carry_val[u];
  y[key] = (T)((double)y[key] + s);
}


}  // namespace spt
