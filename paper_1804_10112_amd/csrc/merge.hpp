// Merge-path machinery shared by the co-iteration kernels (INNERPROD: intersection,
// sparse addition: union) over two ordered, unique COO coordinate lists (Section 4.4).
#pragma once
#include "common.hpp"

namespace spt {

// ---- coordinate keys -------------------------------------------------------
struct Key3 {
  int32_t i, j, k;
};
__device__ __forceinline__ bool key_le(const Key3& a, const Key3& b) {
  if (a.i != b.i) return a.i < b.i;
  if (a.j != b.j) return a.j < b.j;
  return a.k <= b.k;
}
__device__ __forceinline__ bool key_eq(const Key3& a, const Key3& b) {
  return a.i == b.i && a.j == b.j && a.k == b.k;
}
__device__ __forceinline__ bool key_le(uint64_t a, uint64_t b) { return a <= b; }
__device__ __forceinline__ bool key_eq(uint64_t a, uint64_t b) { return a == b; }

// Loaders turn position p of a COO operand into a key. a2 == nullptr for matrices.
struct PackedLoader {
  typedef uint64_t Key;
  const int32_t *a0, *a1, *a2;
  int s0, s1;  // shifts of the first and second coordinate
  __device__ __forceinline__ Key load(int p) const {
    uint64_t k = (static_cast<uint64_t>(static_cast<uint32_t>(a0[p])) << s0) |
                 (static_cast<uint64_t>(static_cast<uint32_t>(a1[p])) << s1);
    if (a2) k |= static_cast<uint32_t>(a2[p]);
    return k;
  }
  __device__ __forceinline__ static Key none() { return ~0ull; }
};
struct TripleLoader {
  typedef Key3 Key;
  const int32_t *a0, *a1, *a2;
  __device__ __forceinline__ Key load(int p) const {
    Key3 k;
    k.i = a0[p];
    k.j = a1[p];
    k.k = a2 ? a2[p] : 0;
    return k;
  }
  __device__ __forceinline__ static Key none() { return Key3{-1, -1, -1}; }
};

// Number of B entries among the first d entries of the merge of B and C (ties: B
// first). The predicate "B[x] precedes C[d-1-x]" is true for small x and false for
// large x; the answer is the first x where it fails. Plain bisection, one lane per
// diagonal: tens of thousands of diagonals are searched at once, and their first
// probes fall on the same few cache lines.
template <typename KL>
__device__ __forceinline__ int merge_path(const KL& kb, const KL& kc, int nb, int nc, int64_t d) {
  int lo = static_cast<int>(d > nc ? d - nc : 0);
  int hi = static_cast<int>(d < nb ? d : nb);
  while (lo < hi) {
    const int mid = lo + ((hi - lo) >> 1);
    if (key_le(kb.load(mid), kc.load(static_cast<int>(d - 1 - mid)))) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// xs[t] = merge-path crossing of the first diagonal of tile t, t = 0..ntiles.
template <typename KL>
__global__ __launch_bounds__(kBlock) void merge_partition_kernel(const KL kb, const KL kc, int nb,
                                                                 int nc, int ntiles, int tile,
                                                                 int* __restrict__ xs) {
  const int t = blockIdx.x * kBlock + threadIdx.x;
  if (t > ntiles) return;
  const int64_t total = static_cast<int64_t>(nb) + nc;
  int64_t d = static_cast<int64_t>(t) * tile;
  if (d > total) d = total;
  xs[t] = merge_path(kb, kc, nb, nc, d);
}

inline int key_bits_of(int64_t extent) {
  int b = 1;
  while (b < 63 && (int64_t{1} << b) < extent) ++b;
  return b;
}

}  // namespace spt
