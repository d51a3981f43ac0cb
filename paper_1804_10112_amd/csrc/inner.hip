// INNERPROD alpha = sum_ijk B_ijk C_ijk (Section 5.3) on two ordered COO tensors, gfx950.
//
// Both operands are ordered and unique, so their coordinate streams are
// intersected with the two-way merge of Section 4.4. One serial merge is a single
// dependency chain; here the merged sequence of nb + nc coordinates is cut into
// equal tiles along its diagonals (a tile is 1792 consecutive steps of the merge,
// whatever mix of B and C entries those are), so the work per workgroup and per
// lane is the same for any ratio of densities and any skew:
//   1. a first kernel finds where every tile's first diagonal crosses the merge
//      path (bisection, one lane per tile);
//   2. the tile's B and C coordinates are staged in LDS, packed into one 64-bit
//      key per entry when the dimensions fit 63 bits;
//   3. every lane finds its own 7-step piece of the path by bisection in LDS and
//      walks it; a C entry that equals the B entry taken just before it is a
//      shared coordinate, noted in LDS;
//   4. the values of the shared coordinates, and only those, are loaded with
//      all lanes side by side and multiplied.
// Ties take the B entry first, so a shared coordinate is seen exactly once, when
// its C entry is taken, also when the two entries fall into different pieces.
// Products are added in double in a fixed order (lane-strided over a tile's C
// entries, shuffle tree, wave order, tile order): the result is reproducible bit for bit.
#include "common.hpp"
#include "merge.hpp"

namespace spt {

constexpr int kIpVT = 7;                   // merge steps per lane: 18 KB of LDS, 8 workgroups per CU
constexpr int kIpTile = kBlock * kIpVT;    // merge steps per tile
constexpr int kIpMaxGrid = 4096;           // workgroups (and partial sums); tiles beyond are looped

template <typename T, typename KL>
__global__ __launch_bounds__(kBlock) void innerprod_kernel(const KL kb, const KL kc,
                                                           const T* __restrict__ bv,
                                                           const T* __restrict__ cv, int nb,
                                                           int nc, int ntiles,
                                                           const int* __restrict__ xs,
                                                           double* __restrict__ partial) {
  typedef typename KL::Key Key;
  // sK[0] = the B entry before the tile (or none), then the tile's B entries, then its C entries
  __shared__ Key sK[kIpTile + 2];  // one spare slot: the walk reads one entry ahead
  __shared__ uint16_t sM[kIpTile];  // per C entry of the tile: 1 + tile index of its B twin
  __shared__ double s_wave[kBlock / kWave];
  constexpr uint16_t kNoTwin = 0xFFFF;

  const int64_t total = static_cast<int64_t>(nb) + nc;
  double acc = 0.0;
  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
  const int64_t d0 = static_cast<int64_t>(tile) * kIpTile;
  const int64_t d1 = d0 + kIpTile < total ? d0 + kIpTile : total;
  const int x0 = xs[tile], x1 = xs[tile + 1];
  const int y0 = static_cast<int>(d0 - x0);
  const int nbl = x1 - x0, ncl = static_cast<int>(d1 - d0) - nbl;
  for (int q = threadIdx.x; q <= nbl; q += kBlock)
    sK[q] = (x0 + q > 0) ? kb.load(x0 + q - 1) : KL::none();
  Key* sC = sK + nbl + 1;
  for (int q = threadIdx.x; q < ncl; q += kBlock) sC[q] = kc.load(y0 + q);
  __syncthreads();
  const Key* sB = sK + 1;  // sB[-1] is the entry before the tile

  const int span = nbl + ncl;
  const int dt = min(static_cast<int>(threadIdx.x) * kIpVT, span);
  const int dend = min(dt + kIpVT, span);
  int lo = dt > ncl ? dt - ncl : 0, hi = dt < nbl ? dt : nbl;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (key_le(sB[mid], sC[dt - 1 - mid])) lo = mid + 1; else hi = mid;
  }
  int x = lo, y = dt - lo;
  // The walk keeps the heads of both lists and the last B entry taken in registers
  // and reads one new key per step (the entry read past either list's end is unused).
  Key prev_b = sB[x - 1], head_b = sB[x], head_c = sC[y];
  for (int s = dt; s < dend; ++s) {
    const bool take_b = y >= ncl || (x < nbl && key_le(head_b, head_c));
    if (take_b) {
      prev_b = head_b;
      head_b = sB[++x];
    } else {
      sM[y] = key_eq(prev_b, head_c) ? static_cast<uint16_t>(x) : kNoTwin;
      head_c = sC[++y];
    }
  }
  __syncthreads();
  // Values of the shared coordinates, loaded side by side after the walk: C's are
  // consecutive over the lanes, B's ascend with them.
#pragma unroll 4
  for (int q = threadIdx.x; q < ncl; q += kBlock) {
    const uint16_t m = sM[q];
    const bool twin = m != kNoTwin;
    const T b = twin ? bv[x0 + m - 1] : T(0);
    const T c = twin ? cv[y0 + q] : T(0);
    acc += static_cast<double>(b) * static_cast<double>(c);
  }
  __syncthreads();  // the next tile overwrites the LDS arrays
  }
  for (int d = kWave / 2; d > 0; d >>= 1) acc += __shfl_down(acc, d, kWave);
  if (lane_id() == 0) s_wave[wave_id()] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < kBlock / kWave; ++w) t += s_wave[w];
    partial[blockIdx.x] = t;
  }
}

// One workgroup adds the tile sums: lane-strided, then the same trees.
template <typename T>
__global__ __launch_bounds__(kBlock) void innerprod_final_kernel(const double* __restrict__ partial,
                                                                 int n, T* __restrict__ out) {
  __shared__ double s_wave[kBlock / kWave];
  double acc = 0.0;
  for (int p = threadIdx.x; p < n; p += kBlock) acc += partial[p];
  for (int d = kWave / 2; d > 0; d >>= 1) acc += __shfl_down(acc, d, kWave);
  if (lane_id() == 0) s_wave[wave_id()] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < kBlock / kWave; ++w) t += s_wave[w];
    *out = static_cast<T>(t);
  }
}

// Fixed: the partial sums plus one crossing per tile for the longest merge that int32
// positions allow (2^32 steps), about 4.6 MB, whatever the operands are.
size_t innerprod_workspace(int64_t) {
  const size_t max_tiles = (size_t{1} << 32) / kIpTile + 2;
  return align_up(kIpMaxGrid * sizeof(double), 256) + align_up(max_tiles * sizeof(int), 256);
}

template <typename T>
static spt_status innerprod_typed(const spt_tensor* B, const spt_tensor* C, void* out, void* ws,
                                  size_t ws_bytes, hipStream_t s) {
  const int nb = static_cast<int>(B->nvals), nc = static_cast<int>(C->nvals);
  const bool any = nb > 0 && nc > 0;
  const int64_t total = static_cast<int64_t>(nb) + nc;
  const int ntiles = any ? static_cast<int>((total + kIpTile - 1) / kIpTile) : 0;
  const int grid = ntiles < kIpMaxGrid ? ntiles : kIpMaxGrid;
  Workspace W(ws, ws_bytes);
  double* partial = W.take<double>(grid > 0 ? grid : 1);
  int* xs = W.take<int>(static_cast<size_t>(ntiles) + 1);
  if (ntiles > 0 && (!ws || !W.ok()))
    return fail(SPT_ERR_WORKSPACE, "innerprod: workspace of %zu bytes, %zu needed", ws_bytes,
                W.used);
  const bool third = B->order == 3;
  const int32_t* b2 = third ? B->level[2].crd : nullptr;
  const int32_t* c2 = third ? C->level[2].crd : nullptr;
  const T* bv = static_cast<const T*>(B->vals);
  const T* cv = static_cast<const T*>(C->vals);
  if (ntiles > 0) {
    const int pgrid = (ntiles + 1 + kBlock - 1) / kBlock;
    const int w1 = key_bits_of(B->level[1].N), w2 = third ? key_bits_of(B->level[2].N) : 0;
    if (key_bits_of(B->level[0].N) + w1 + w2 <= 63) {
      PackedLoader kb{B->level[0].crd, B->level[1].crd, b2, w1 + w2, w2};
      PackedLoader kc{C->level[0].crd, C->level[1].crd, c2, w1 + w2, w2};
      hipLaunchKernelGGL(merge_partition_kernel<PackedLoader>, dim3(pgrid), dim3(kBlock), 0, s, kb, kc,
                         nb, nc, ntiles, kIpTile, xs);
      hipLaunchKernelGGL((innerprod_kernel<T, PackedLoader>), dim3(grid), dim3(kBlock), 0, s, kb,
                         kc, bv, cv, nb, nc, ntiles, xs, partial);
    } else {
      TripleLoader kb{B->level[0].crd, B->level[1].crd, b2};
      TripleLoader kc{C->level[0].crd, C->level[1].crd, c2};
      hipLaunchKernelGGL(merge_partition_kernel<TripleLoader>, dim3(pgrid), dim3(kBlock), 0, s, kb, kc,
                         nb, nc, ntiles, kIpTile, xs);
      hipLaunchKernelGGL((innerprod_kernel<T, TripleLoader>), dim3(grid), dim3(kBlock), 0, s, kb,
                         kc, bv, cv, nb, nc, ntiles, xs, partial);
    }
    SPT_CHECK_LAUNCH("innerprod");
  }
  hipLaunchKernelGGL(innerprod_final_kernel<T>, dim3(1), dim3(kBlock), 0, s, partial, grid,
                     static_cast<T*>(out));
  SPT_CHECK_LAUNCH("innerprod final");
  return SPT_OK;
}

spt_status innerprod_dispatch(Format, const spt_tensor* B, const spt_tensor* C, void* out,
                              void* ws, size_t ws_bytes, hipStream_t s) {
  return B->dtype == SPT_F64 ? innerprod_typed<double>(B, C, out, ws, ws_bytes, s)
                             : innerprod_typed<float>(B, C, out, ws, ws_bytes, s);
}

}  // namespace spt
