// spt_validate: device-side check of what the other entry points take on trust -- the CONTENT
// of the level arrays (Section 3.1): pos of a compressed level starts at 0, never decreases
// and ends at the number of positions of its level; stored coordinates lie inside their
// dimension (-1 marks padding in singleton and hashed levels); a level flagged ordered /
// unique really stores ascending / strictly ascending coordinates inside every segment, and a
// COO tensor flagged ordered on all levels is in lexicographic order. Nothing is synchronised:
// the verdict is written to device memory.
#include "common.hpp"

namespace spt {

enum : int32_t {
  kBadPosStart = 1,   // pos[0] != 0 or pos decreases
  kBadPosEnd = 2,     // pos[last] != number of positions of the level
  kBadCrd = 4,        // coordinate outside [0, N) (or below -1 where padding is allowed)
  kBadOrder = 8,      // ordered / unique flag violated
  kBadOffset = 16     // offset of a range / offset level moves every coordinate out of range
};

__device__ __forceinline__ void report(int32_t* err, int32_t kind) {
  atomicAdd(&err[0], 1);
  atomicOr(&err[1], kind);
}

__global__ void validate_init_kernel(int32_t* err) {
  if (threadIdx.x == 0 && blockIdx.x == 0) err[0] = err[1] = 0;
}

// pos[0 .. M]: starts at 0, monotone, ends at `count`.
__global__ __launch_bounds__(kBlock) void validate_pos_kernel(int64_t M, int64_t count,
                                                              const int32_t* __restrict__ pos,
                                                              int32_t* __restrict__ err) {
  const int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (q > M) return;
  const int32_t v = pos[q];
  if (q == 0 && v != 0) report(err, kBadPosStart);
  if (q < M && pos[q + 1] < v) report(err, kBadPosStart);
  if (q == M && v != count) report(err, kBadPosEnd);
}

// crd[p * stride], p < n: inside [lowest, N).
__global__ __launch_bounds__(kBlock) void validate_crd_kernel(int64_t n, int64_t stride, int64_t N,
                                                              int32_t lowest,
                                                              const int32_t* __restrict__ crd,
                                                              int32_t* __restrict__ err) {
  const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (p >= n) return;
  const int32_t c = crd[p * stride];
  if (c < lowest || c >= N) report(err, kBadCrd);
}

// Inside every segment of a compressed level the coordinates ascend (strictly if unique).
// A descent between p - 1 and p is legal only where p starts a segment, i.e. where p is an
// entry of pos (looked up by bisection, only at descents).
__global__ __launch_bounds__(kBlock) void validate_segment_order_kernel(
    int64_t n, int64_t M, int strict, const int32_t* __restrict__ pos, const int32_t* __restrict__ crd,
    int32_t* __restrict__ err) {
  const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (p < 1 || p >= n) return;
  const int32_t a = crd[p - 1], b = crd[p];
  if (a < b || (!strict && a == b)) return;
  int64_t lo = 0, hi = M + 1;  // first q with pos[q] >= p
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (pos[mid] < p) lo = mid + 1; else hi = mid;
  }
  if (lo > M || pos[lo] != p) report(err, kBadOrder);
}

// COO flagged ordered on every level: entries in lexicographic order of (c0, c1[, c2]).
__global__ __launch_bounds__(kBlock) void validate_coo_order_kernel(int64_t n, int order,
                                                                    const int32_t* __restrict__ c0,
                                                                    const int32_t* __restrict__ c1,
                                                                    const int32_t* __restrict__ c2,
                                                                    int32_t* __restrict__ err) {
  const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (p < 1 || p >= n) return;
  bool less = false, greater = false;
  const int32_t* c[3] = {c0, c1, c2};
  for (int m = 0; m < order && !less && !greater; ++m) {
    const int32_t a = c[m][p - 1], b = c[m][p];
    less = a < b;
    greater = a > b;
  }
  if (greater) report(err, kBadOrder);
}

// offset[d], d < K: some row of the range level must keep its column inside [0, M).
__global__ __launch_bounds__(kBlock) void validate_offset_kernel(int64_t K, int64_t N, int64_t M,
                                                                 const int32_t* __restrict__ offset,
                                                                 int32_t* __restrict__ err) {
  const int64_t d = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (d >= K) return;
  const int64_t off = offset[d];
  if (off <= -N || off >= M) report(err, kBadOffset);
}

static unsigned grid_for(int64_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

// T has passed the host checks (recognize() / generic_ok()): kinds, pointers and sizes are sane.
spt_status validate_dispatch(const spt_tensor* T, int32_t* err, hipStream_t s) {
  hipLaunchKernelGGL(validate_init_kernel, dim3(1), dim3(kWave), 0, s, err);
  SPT_CHECK_LAUNCH("validate init");
  const spt_level* L = T->level;
  const int nl = T->nlevels;
  // positions per level, from the values backwards: the last level has nvals positions; a
  // singleton / offset level has as many as its parent, a dense / range / hashed level N (W)
  // per parent, a compressed level declares its parent count in M
  int64_t P[5];  // P[k + 1] = positions of level k, P[0] = positions above level 0 (one root)
  P[nl] = T->nvals;
  for (int k = nl - 1; k >= 0; --k) {
    const int64_t per = L[k].kind == SPT_HASHED ? L[k].M : L[k].N;
    switch (L[k].kind) {
      case SPT_COMPRESSED: P[k] = L[k].M; break;
      case SPT_SINGLETON:
      case SPT_OFFSET: P[k] = P[k + 1]; break;
      default:
        if (per <= 0 || P[k + 1] % per != 0)
          return P[k + 1] == 0 && per >= 0
                     ? SPT_OK
                     : fail(SPT_ERR_INVALID_ARG,
                            "validate: level %d: %lld positions are no multiple of the level's extent %lld", k,
                            (long long)P[k + 1], (long long)per);
        P[k] = P[k + 1] / per;
    }
  }
  if (P[0] != 1)
    return fail(SPT_ERR_INVALID_ARG, "validate: the level sizes imply %lld root positions instead of 1",
                (long long)P[0]);
  bool coo_ordered = L[0].kind == SPT_COMPRESSED && nl >= 2 && (L[0].flags & SPT_ORDERED);
  for (int k = 0; k < nl; ++k) {
    const int64_t n = P[k + 1], stride = L[k].crd_stride > 1 ? L[k].crd_stride : 1;
    if (k > 0 && !(L[k].kind == SPT_SINGLETON && (L[k].flags & SPT_ORDERED))) coo_ordered = false;
    if (n >= INT32_MAX || P[k] >= INT32_MAX)
      return fail(SPT_ERR_UNSUPPORTED, "validate: level %d has more than 2^31 positions", k);
    if (L[k].kind == SPT_COMPRESSED) {
      hipLaunchKernelGGL(validate_pos_kernel, dim3(grid_for(P[k] + 1)), dim3(kBlock), 0, s, P[k], n, L[k].pos, err);
      SPT_CHECK_LAUNCH("validate pos");
    }
    const bool stored = L[k].kind == SPT_COMPRESSED || L[k].kind == SPT_SINGLETON || L[k].kind == SPT_HASHED;
    if (stored && n > 0) {
      const int32_t lowest = L[k].kind == SPT_COMPRESSED ? 0 : -1;
      hipLaunchKernelGGL(validate_crd_kernel, dim3(grid_for(n)), dim3(kBlock), 0, s, n, stride, L[k].N, lowest,
                         L[k].crd, err);
      SPT_CHECK_LAUNCH("validate crd");
    }
    // a compressed level below the root: its flags speak about each segment
    if (L[k].kind == SPT_COMPRESSED && (L[k].flags & SPT_ORDERED) && stride == 1 && n > 1 &&
        !(k == 0 && nl >= 2 && L[1].kind == SPT_SINGLETON)) {
      hipLaunchKernelGGL(validate_segment_order_kernel, dim3(grid_for(n)), dim3(kBlock), 0, s, n, P[k],
                         (L[k].flags & SPT_UNIQUE) ? 1 : 0, L[k].pos, L[k].crd, err);
      SPT_CHECK_LAUNCH("validate order");
    }
    // DIA shape (dense diagonals, range rows, ...): the range level's offsets, one per diagonal
    if (L[k].kind == SPT_RANGE && k == 1 && L[0].kind == SPT_DENSE && L[0].N > 0) {
      hipLaunchKernelGGL(validate_offset_kernel, dim3(grid_for(L[0].N)), dim3(kBlock), 0, s, L[0].N, L[k].N,
                         L[k].M, L[k].offset, err);
      SPT_CHECK_LAUNCH("validate offset");
    }
  }
  if (coo_ordered && T->nvals > 1 && nl <= 3) {
    bool contiguous = true;
    for (int k = 0; k < nl; ++k) contiguous = contiguous && L[k].crd_stride <= 1;
    if (contiguous) {
      hipLaunchKernelGGL(validate_coo_order_kernel, dim3(grid_for(T->nvals)), dim3(kBlock), 0, s, T->nvals, nl,
                         L[0].crd, L[1].crd, nl > 2 ? L[2].crd : nullptr, err);
      SPT_CHECK_LAUNCH("validate coo order");
    }
  }
  return SPT_OK;
}

}  // namespace spt
