// SpMV on UNORDERED COO without one global atomic per entry.
//
// The paper's COO kernel is a single fused loop that scatters v*x[j] into y
// (Section 4.5, fusing iterators; Section 5.2.1). A literal GPU version issues
// one floating-point atomic per stored entry at a random address, which the
// memory system serves at only ~15 G atomics/s. Here the scatter is split in
// two coalesced steps:
//   1. bin: one pass of the radix machinery on the top 8 bits of the row moves
//      (row, v*x[col]) into 256 row-range bins (histogram, scan, stable scatter);
//      the gather of x happens here, once per entry.
//   2. accumulate: a workgroup owns a slice of one bin's entries and a sub-range
//      of the bin's rows that fits LDS (128 KB: usually the whole bin), adds the products with LDS atomics and
//      writes its rows: plain stores when it holds the whole bin, otherwise
//      atomics onto the zero-filled y (one per touched row and slice).
// Like the atomic kernel the result is order-dependent in the last bits
// (tolerance-checked, not bit-reproducible); the ordered COO path is exact-order.
#include "common.hpp"
#include "radix.hpp"
#include "scan.hpp"

namespace spt {

template <typename T>
__device__ __forceinline__ T ld_nt(const T* p) {
  return __builtin_nontemporal_load(p);
}

// Stable scatter by bin = (row >> shift) & 255 of (row, vals * x[col]); the same
// ranking and in-LDS tile sort as the sort's scatter kernel.
template <typename T>
__global__ __launch_bounds__(kBlock) void bin_scatter_kernel(
    int n, int shift, int ntiles, const int32_t* __restrict__ off, const int32_t* __restrict__ row,
    const int32_t* __restrict__ col, const T* __restrict__ vals, const T* __restrict__ x,
    int32_t* __restrict__ brow, T* __restrict__ bprod) {
  __shared__ int s_cnt[kWaves][kRadix];
  __shared__ int s_gdelta[kRadix];
  __shared__ T s_buf[kSortTile];
  int32_t* s_buf32 = reinterpret_cast<int32_t*>(s_buf);
  const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
  const int tile = xcd_contiguous_block_id();
  for (int q = tid; q < kWaves * kRadix; q += kBlock) (&s_cnt[0][0])[q] = 0;
  __syncthreads();
  const int tile_base = tile * kSortTile;
  const int tile_n = min(kSortTile, n - tile_base);
  const int wave_base = tile_base + w * (kWave * kSortIPT);
  const uint64_t lanes_below = ((uint64_t)1 << lane) - 1;
  volatile int* cnt = s_cnt[w];

  int32_t key[kSortIPT];
  T prod[kSortIPT];
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {
    const int i = wave_base + k * kWave + lane;
    const bool valid = i < n;
    key[k] = valid ? ld_nt(row + i) : 0;
    prod[k] = valid ? ld_nt(vals + i) * x[ld_nt(col + i)] : T(0);
  }
  int lpos[kSortIPT];
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {
    const bool valid = wave_base + k * kWave + lane < n;
    const int d = digit_of(key[k], shift);
    uint64_t same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < kRadixBits; ++b) {
      const bool bit = (d >> b) & 1;
      const uint64_t vote = __ballot(valid && bit);
      same &= bit ? vote : ~vote;
    }
    const int before = __popcll(same & lanes_below);
    int basecnt = 0;
    if (valid) basecnt = cnt[d];
    __builtin_amdgcn_wave_barrier();
    if (valid && before == 0) cnt[d] = basecnt + __popcll(same);
    __builtin_amdgcn_wave_barrier();
    lpos[k] = basecnt + before;
  }
  __syncthreads();
  {
    const int d = tid;
    int c[kWaves], tot = 0;
#pragma unroll
    for (int u = 0; u < kWaves; ++u) {
      c[u] = s_cnt[u][d];
      tot += c[u];
    }
    int all;
    int start = block_inclusive_sum(tot, &all) - tot;
    s_gdelta[d] = off[(int64_t)d * ntiles + tile] - start;
#pragma unroll
    for (int u = 0; u < kWaves; ++u) {
      s_cnt[u][d] = start;
      start += c[u];
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {
    if (wave_base + k * kWave + lane < n) {
      lpos[k] += s_cnt[w][digit_of(key[k], shift)];
      s_buf32[lpos[k]] = key[k];
    }
  }
  __syncthreads();
  int dst[kSortIPT];
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {
    const int j = k * kBlock + tid;
    if (j < tile_n) {
      const int32_t kk = s_buf32[j];
      dst[k] = j + s_gdelta[digit_of(kk, shift)];
      brow[dst[k]] = kk;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k)
    if (wave_base + k * kWave + lane < n) s_buf[lpos[k]] = prod[k];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {
    const int j = k * kBlock + tid;
    if (j < tile_n) bprod[dst[k]] = s_buf[j];
  }
}

// Work item = (bin b, slice k of the bin's entries, row sub-range sub).
// kBinSlice entries per slice; RB rows per LDS accumulator.
constexpr int kBinSlice = 1 << 18;

template <typename T>
struct BinRows {
  // 128 KB of the CU's 160 KB LDS: with 256 bins every matrix of up to 2^22 (fp64) or 2^23
  // (fp32) rows has a single sub-range, so each binned entry is read exactly once
  static constexpr int value = 131072 / sizeof(T);
};

constexpr int kAccBlock = 1024;  // one workgroup streams a whole slice: it needs many loads in flight

template <typename T>
__global__ __launch_bounds__(kAccBlock) void bin_accumulate_kernel(
    int n, int shift, int ntiles, int nsub, const int32_t* __restrict__ off,
    const int32_t* __restrict__ brow, const T* __restrict__ bprod, int nrows, T* __restrict__ y) {
  constexpr int RB = BinRows<T>::value;
  __shared__ T s_acc[RB];
  __shared__ int s_start[kRadix + 1];
  __shared__ int s_segbase[kRadix + 1];
  const int tid = threadIdx.x;
  const int item = blockIdx.x / nsub, sub = blockIdx.x % nsub;

  if (tid < kRadix) s_start[tid] = off[(int64_t)tid * ntiles];  // first position of bin tid
  if (tid == 0) s_start[kRadix] = n;
  __syncthreads();
  if (tid == 0) {  // slices per bin, running sum
    int run = 0;
    for (int q = 0; q < kRadix; ++q) {
      s_segbase[q] = run;
      run += (s_start[q + 1] - s_start[q] + kBinSlice - 1) / kBinSlice;
    }
    s_segbase[kRadix] = run;
  }
  __syncthreads();
  if (item >= s_segbase[kRadix]) return;  // uniform: the grid is an upper bound on the item count
  int b = 0;  // the bin whose slice range contains item (every thread searches, 8 steps)
  for (int step = kRadix / 2; step > 0; step >>= 1)
    if (s_segbase[b + step] <= item) b += step;
  const int k = item - s_segbase[b];
  const int begin = s_start[b] + k * kBinSlice;
  const int end = min(begin + kBinSlice, s_start[b + 1]);
  const bool whole_bin = (s_segbase[b + 1] - s_segbase[b]) == 1;
  const int64_t r0 = ((int64_t)b << shift) + (int64_t)sub * RB;  // first row of this sub-range
  const int64_t rows_in_bin = (int64_t)1 << shift;
  const int nr = (int)min<int64_t>(RB, rows_in_bin - (int64_t)sub * RB);

  for (int q = tid; q < nr; q += kAccBlock) s_acc[q] = T(0);
  __syncthreads();
  // software pipeline: the loads of batch i+1 are in flight while batch i is accumulated
  constexpr int U = 4;
  int32_t r[U], rn[U];
  T v[U], vn[U];
  auto load = [&](int p0, int32_t* rr, T* vv) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int p = p0 + u * kAccBlock;
      rr[u] = p < end ? ld_nt(brow + p) : -1;
      vv[u] = p < end ? ld_nt(bprod + p) : T(0);
    }
  };
  load(begin + tid, r, v);
  for (int p0 = begin + tid; p0 < end; p0 += kAccBlock * U) {
    load(p0 + kAccBlock * U, rn, vn);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = (int64_t)r[u] - r0;
      if (r[u] >= 0 && q >= 0 && q < nr) atomicAdd(&s_acc[q], v[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      r[u] = rn[u];
      v[u] = vn[u];
    }
  }
  __syncthreads();
  for (int q = tid; q < nr; q += kAccBlock) {
    const int64_t rr = r0 + q;
    if (rr < nrows) {
      const T a = s_acc[q];
      if (whole_bin) y[rr] = a;
      else if (a != T(0)) unsafeAtomicAdd(y + rr, a);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void zero_t_kernel(T* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) out[i] = T(0);
}

struct BinPlan {
  int ntiles, shift, nsub;
  size_t total;
};

template <typename T>
static BinPlan bin_plan(int64_t nnz, int64_t nrows) {
  BinPlan P;
  P.ntiles = (int)((nnz + kSortTile - 1) / kSortTile);
  const int bits = bits_for(nrows);
  P.shift = bits > kRadixBits ? bits - kRadixBits : 0;
  const int64_t rows_in_bin = (int64_t)1 << P.shift;
  P.nsub = (int)((rows_in_bin + BinRows<T>::value - 1) / BinRows<T>::value);
  P.total = align_up((size_t)nnz * 4, 256) + align_up((size_t)nnz * sizeof(T), 256) +
            align_up((size_t)kRadix * P.ntiles * 4, 256) + scan_workspace((int64_t)kRadix * P.ntiles) +
            256;
  return P;
}

size_t coo_binned_workspace(int dtype, int64_t nnz, int64_t nrows) {
  return dtype == SPT_F64 ? bin_plan<double>(nnz, nrows).total : bin_plan<float>(nnz, nrows).total;
}

template <typename T>
spt_status coo_binned_spmv(int64_t nnz64, int64_t nrows, const int32_t* row, const int32_t* col,
                           const T* vals, const T* x, T* y, void* ws, size_t ws_bytes,
                           hipStream_t s) {
  if (nnz64 + kSortTile >= INT32_MAX || nrows + 1 >= INT32_MAX)
    return fail(SPT_ERR_UNSUPPORTED, "spmv: more than 2^31 entries or rows");
  const int nnz = (int)nnz64;
  const BinPlan P = bin_plan<T>(nnz, nrows);
  if (!ws || ws_bytes < P.total)
    return fail(SPT_ERR_WORKSPACE, "spmv: workspace of %zu bytes needed, %zu given", P.total,
                ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* brow = W.take<int32_t>(nnz);
  T* bprod = W.take<T>(nnz);
  int32_t* hist = W.take<int32_t>((size_t)kRadix * P.ntiles);
  int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace((int64_t)kRadix * P.ntiles)));

  hipLaunchKernelGGL(zero_t_kernel<T>, dim3((unsigned)((nrows + kBlock - 1) / kBlock)), dim3(kBlock),
                     0, s, y, nrows);
  SPT_CHECK_LAUNCH("zero y");
  spt_status st = launch_radix_hist(row, nnz, P.shift, P.ntiles, hist, s);
  if (st != SPT_OK) return st;
  st = device_scan_i32<false>(hist, hist, (int64_t)kRadix * P.ntiles, scan_tmp, s);
  if (st != SPT_OK) return st;
  hipLaunchKernelGGL(bin_scatter_kernel<T>, dim3(P.ntiles), dim3(kBlock), 0, s, nnz, P.shift,
                     P.ntiles, hist, row, col, vals, x, brow, bprod);
  SPT_CHECK_LAUNCH("bin_scatter");
  const int64_t items = (nnz64 + kBinSlice - 1) / kBinSlice + kRadix;  // upper bound
  hipLaunchKernelGGL(bin_accumulate_kernel<T>, dim3((unsigned)(items * P.nsub)), dim3(kAccBlock), 0, s,
                     nnz, P.shift, P.ntiles, P.nsub, hist, brow, bprod, (int)nrows, y);
  SPT_CHECK_LAUNCH("bin_accumulate");
  return SPT_OK;
}

template spt_status coo_binned_spmv<double>(int64_t, int64_t, const int32_t*, const int32_t*,
                                            const double*, const double*, double*, void*, size_t,
                                            hipStream_t);
template spt_status coo_binned_spmv<float>(int64_t, int64_t, const int32_t*, const int32_t*,
                                           const float*, const float*, float*, void*, size_t,
                                           hipStream_t);

}  // namespace spt
