// SpMV y = A x on CSR, COO, DIA and ELL (paper Section 5.2), gfx950.
//
// All four kernels are bound by HBM bandwidth: the matrix arrays are streamed
// once with coalesced (non-temporal) loads, x is gathered through the caches.
//  * CSR and sorted COO share one kernel: a workgroup owns a fixed chunk of
//    stored entries (balanced in entries, not rows, so power-law rows cost
//    nothing extra), stages the products in LDS and reduces them per row with a
//    segmented scan; a row cut by a chunk boundary is finished by a tiny carry
//    kernel. No atomics, results are bit-reproducible.
//  * Unsorted COO is the paper's scatter loop: atomic adds into y.
//  * DIA and ELL read the diagonal-major / slot-major arrays with consecutive
//    rows in consecutive lanes.
#include <algorithm>
#include <cstdlib>

#include "common.hpp"
#include "segreduce.hpp"
#include "wavescan.hpp"

namespace spt {

template <typename T>
__device__ __forceinline__ T ld_stream(const T* p) {
  return __builtin_nontemporal_load(p);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void fill_kernel(T* __restrict__ out, int64_t n, T value) {
  int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) out[i] = value;
}

// ---------------------------------------------------------------- DIA
// Cell (d,i) at d*N+i holds A(i, i+offset[d]) (range level: rows, offset
// level: cols; Table 2). One row per thread, the diagonals in a register loop.
constexpr int kDiaMaxLdsOffsets = 1024;

template <typename T>
__global__ __launch_bounds__(kBlock) void dia_spmv_kernel(int64_t N, int64_t M, int K,
                                                          const int32_t* __restrict__ offset,
                                                          const T* __restrict__ vals,
                                                          const T* __restrict__ x,
                                                          T* __restrict__ y) {
  __shared__ int32_t s_off[kDiaMaxLdsOffsets];
  const bool in_lds = K <= kDiaMaxLdsOffsets;
  if (in_lds) {
    for (int d = threadIdx.x; d < K; d += kBlock) s_off[d] = offset[d];
    __syncthreads();
  }
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= N) return;
  T acc = 0;
#pragma unroll 8
  for (int d = 0; d < K; ++d) {
    const int64_t j = i + (in_lds ? s_off[d] : offset[d]);
    if (j >= 0 && j < M) acc += ld_stream(vals + (int64_t)d * N + i) * x[j];
  }
  y[i] = acc;
}

// ---------------------------------------------------------------- ELL
// Cell (k,i) at k*N+i; a negative column marks padding and is skipped without
// touching its value or x.
template <typename T>
__global__ __launch_bounds__(kBlock) void ell_spmv_kernel(int64_t N, int W,
                                                          const int32_t* __restrict__ crd,
                                                          const T* __restrict__ vals,
                                                          const T* __restrict__ x,
                                                          T* __restrict__ y) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= N) return;
  T acc = 0;
#pragma unroll 8
  for (int k = 0; k < W; ++k) {
    const int32_t j = ld_stream(crd + (int64_t)k * N + i);
    if (j >= 0) acc += ld_stream(vals + (int64_t)k * N + i) * x[j];
  }
  y[i] = acc;
}

// ---------------------------------------------------------------- DIA / ELL, R rows per lane
// Same computations with 16-byte loads: a lane owns R consecutive rows (R = 2
// for fp64, 4 for fp32), so every access to the diagonal-major / slot-major
// arrays is one aligned 16-byte vector. HBM delivers ~7 TB/s to 16-byte lane
// loads but under 4 TB/s to 4-byte ones, hence the width. Needs N % R == 0 and
// 16-byte aligned arrays (checked on the host; otherwise the scalar kernels run).
template <typename T> struct VecOf;
template <> struct VecOf<double> { static constexpr int R = 2; typedef double type __attribute__((ext_vector_type(2))); typedef int32_t itype __attribute__((ext_vector_type(2))); };
template <> struct VecOf<float> { static constexpr int R = 4; typedef float type __attribute__((ext_vector_type(4))); typedef int32_t itype __attribute__((ext_vector_type(4))); };

// KT > 0: the number of diagonals is the compile-time constant KT, so all KT
// diagonal loads and their x loads are issued before the first use (one memory
// round trip per lane). KT == 0: any K, in batches of 8 (the tail batch re-reads
// the last diagonal and masks it out).
// A diagonal whose row range [max(0,-off), min(N, M-off)) misses all rows of the
// wave is skipped by the whole wave (a scalar branch): far diagonals are empty
// over half the matrix, and loading their cells would move bytes that are never
// used. Inside a live wave no load sits behind a per-lane branch: cells outside the
// range are loaded (they are inside the array) and masked, x is read at a clamped
// index. XV: x is 16-byte aligned and M a multiple of R, so a diagonal whose offset
// is a multiple of R reads its R values of x as one aligned 16-byte load.
template <typename T, int KT, bool XV>
__global__ __launch_bounds__(kBlock) void dia_spmv_vec_kernel(int64_t N, int64_t M, int K,
                                                              const int32_t* __restrict__ offset,
                                                              const T* __restrict__ vals,
                                                              const T* __restrict__ x,
                                                              T* __restrict__ y) {
  constexpr int R = VecOf<T>::R;
  constexpr int B = KT > 0 ? KT : 8;
  using V = typename VecOf<T>::type;
  const int64_t blk0 = (int64_t)xcd_contiguous_block_id() * kBlock;
  const int64_t i0 = (blk0 + threadIdx.x) * R;
  // rows [w0, w1) belong to this wave (uniform: kept in scalar registers)
  const int64_t w0 = (blk0 + __builtin_amdgcn_readfirstlane(threadIdx.x & ~(kWave - 1))) * R;
  const int64_t w1 = w0 + kWave * R;
  if (i0 >= N) return;
  V acc = 0;
  const int kend = KT > 0 ? KT : K;
  for (int d0 = 0; d0 < kend; d0 += B) {
    V v[B];
    V xv[B];
    int64_t j0[B];
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int d = min(d0 + u, kend - 1);
      const int64_t off = offset[d];  // uniform address: a scalar load
      j0[u] = i0 + off;
      v[u] = 0;
      xv[u] = 0;
      const int64_t lo = off < 0 ? -off : 0, hi = (M - off) < N ? (M - off) : N;
      if (w0 < hi && w1 > lo) {  // uniform
        v[u] = ld_stream(reinterpret_cast<const V*>(vals + (int64_t)d * N + i0));
        if (XV && (off % R) == 0) {  // uniform; j0 is a multiple of R
          const int64_t jc = j0[u] < 0 ? 0 : (j0[u] > M - R ? M - R : j0[u]);
          xv[u] = *reinterpret_cast<const V*>(x + jc);
        } else {
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const int64_t j = j0[u] + r;
            xv[u][r] = x[j < 0 ? 0 : (j >= M ? M - 1 : j)];
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < B; ++u) {
      if (d0 + u < kend) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const int64_t j = j0[u] + r;
          acc[r] += (j >= 0 && j < M) ? v[u][r] * xv[u][r] : T(0);
        }
      }
    }
  }
  *reinterpret_cast<V*>(y + i0) = acc;
}

// Bound by the gathers of x (one cache line per stored entry), so the loop is
// kept simple: padding neither gathers nor multiplies.
template <typename T>
__global__ __launch_bounds__(kBlock) void ell_spmv_vec_kernel(int64_t N, int W,
                                                              const int32_t* __restrict__ crd,
                                                              const T* __restrict__ vals,
                                                              const T* __restrict__ x,
                                                              T* __restrict__ y) {
  constexpr int R = VecOf<T>::R;
  using V = typename VecOf<T>::type;
  using IV = typename VecOf<T>::itype;
  const int64_t i0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * R;
  if (i0 >= N) return;
  V acc = 0;
#pragma unroll 4
  for (int k = 0; k < W; ++k) {
    const IV j = ld_stream(reinterpret_cast<const IV*>(crd + (int64_t)k * N + i0));
    const V v = ld_stream(reinterpret_cast<const V*>(vals + (int64_t)k * N + i0));
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (j[r] >= 0) acc[r] += v[r] * x[j[r]];
  }
  *reinterpret_cast<V*>(y + i0) = acc;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// ---------------------------------------------------------------- CSR / sorted COO
// Chunk of IPT*256 consecutive entries per workgroup.
//   phase 1  coalesced load of col/vals (and row for COO), gather x, product
//            and key into LDS (padded so that phase 2 is bank-conflict free)
//   CSR only the rows that start inside the chunk are found with two wave-wide
//            searches of pos; each such row marks its first entry as a head
//            (empty rows store y = 0 directly)
//   phase 2  every thread reduces IPT consecutive entries, segments that start
//            and end inside one thread are stored at once; a workgroup scan of
//            the per-thread summaries closes the rest
// Output protocol: the workgroup that contains a row's first entry stores the
// row's (possibly partial) sum with a plain store; the sum of the entries that
// precede the first head of a chunk leaves as carry (key, value) number
// `chunk`, key -1 if there is none.
template <int IPT>
__device__ __forceinline__ int lds_slot(int e) { return e + e / IPT; }

// How an entry's column is turned into x_j ("locate" into the vector operand,
// Section 3.2): a dense array, an ordered sparse vector (binary search of its
// crd), or a hash-map vector (Table 2's probing: start at j % W, step +1 with
// wrap, stop at j, at an empty bucket (-1) or after a full cycle).
template <typename T>
struct DenseX {
  const T* __restrict__ x;
  __device__ __forceinline__ T at(int32_t j) const { return x[j]; }
};
template <typename T>
struct SparseX {
  const int32_t* __restrict__ crd;
  const T* __restrict__ vals;
  int n;
  __device__ __forceinline__ T at(int32_t j) const {
    int lo = 0, hi = n;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (crd[mid] < j) lo = mid + 1;
      else hi = mid;
    }
    return (lo < n && crd[lo] == j) ? vals[lo] : T(0);
  }
};
template <typename T>
struct HashX {
  const int32_t* __restrict__ crd;
  const T* __restrict__ vals;
  int W;
  __device__ __forceinline__ T at(int32_t j) const {
    int p = j % W;
    for (int step = 0; step < W; ++step) {
      const int32_t c = crd[p];
      if (c == j) return vals[p];
      if (c == -1) break;
      p = p + 1 == W ? 0 : p + 1;
    }
    return T(0);
  }
};

template <typename T, bool CSR, int IPT, bool VEC, class XP = DenseX<T>>
__global__ __launch_bounds__(kBlock) void seg_spmv_kernel(
    int nnz, int nrows, const int32_t* __restrict__ pos_or_row, const int32_t* __restrict__ col,
    const T* __restrict__ vals, const XP x, T* __restrict__ y,
    int32_t* __restrict__ carry_key, T* __restrict__ carry_val,
    const int32_t* __restrict__ select, int want) {
  constexpr int CHUNK = IPT * kBlock;
  if (!selected(select, want)) return;  // the other CSR kernel was chosen on the device
  __shared__ T s_val[CHUNK + kBlock];
  __shared__ int32_t s_key[CHUNK + kBlock];
  __shared__ SegScanStorage<T> s_scan;
  __shared__ int s_rows[2];

  const int tid = threadIdx.x;
  const int chunk = xcd_contiguous_block_id();
  const int base = chunk * CHUNK;  // host guarantees nnz + CHUNK < 2^31
  const int end = min(base + CHUNK, nnz);
  const bool last_chunk = (end == nnz);

  if (CSR) {
    if (wave_id() == 0) {
      int r = wave_lower_bound(pos_or_row, nrows + 1, base);
      if (lane_id() == 0) s_rows[0] = r;
    } else if (wave_id() == 1) {
      int r = last_chunk ? nrows : wave_lower_bound(pos_or_row, nrows + 1, end);
      if (lane_id() == 0) s_rows[1] = r;
    }
  }

  // phase 1: a lane loads R consecutive entries per step with 16-byte (fp32) or
  // 8+16-byte (fp64) vector loads when the arrays allow it
  constexpr int R = VecOf<T>::R;
  using V = typename VecOf<T>::type;
  using IV = typename VecOf<T>::itype;
  int32_t fill_key = -1;
  if (!CSR) fill_key = pos_or_row[end - 1];  // tail padding extends the last segment
#pragma unroll
  for (int q = 0; q < IPT / R; ++q) {
    const int e0 = (q * kBlock + tid) * R;
    const int p0 = base + e0;
    int32_t c[R], key[R];
    T v[R];
    bool ok[R];
    if (VEC && p0 + R <= end) {
      const IV cv = ld_stream(reinterpret_cast<const IV*>(col + p0));
      const V vv = ld_stream(reinterpret_cast<const V*>(vals + p0));
      IV kv = fill_key;
      if (!CSR) kv = ld_stream(reinterpret_cast<const IV*>(pos_or_row + p0));
#pragma unroll
      for (int r = 0; r < R; ++r) {
        c[r] = cv[r];
        v[r] = vv[r];
        key[r] = kv[r];
        ok[r] = true;
      }
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        ok[r] = p0 + r < end;
        c[r] = ok[r] ? ld_stream(col + p0 + r) : 0;
        v[r] = ok[r] ? ld_stream(vals + p0 + r) : T(0);
        key[r] = (!CSR && ok[r]) ? ld_stream(pos_or_row + p0 + r) : fill_key;
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      s_val[lds_slot<IPT>(e0 + r)] = ok[r] ? v[r] * x.at(c[r]) : T(0);
      s_key[lds_slot<IPT>(e0 + r)] = key[r];
    }
  }
  int32_t prev_key = -1;  // key of the entry before the chunk (COO)
  if (!CSR && base > 0) prev_key = pos_or_row[base - 1];
  __syncthreads();

  int carry_row = prev_key;
  if (CSR) {
    const int r_lo = s_rows[0], r_hi = s_rows[1];
    // the row cut by the chunk start, if the chunk does not begin with a head
    carry_row = r_lo - 1;
    for (int r = r_lo + tid; r < r_hi; r += kBlock) {
      const int a = pos_or_row[r], b = pos_or_row[r + 1];
      if (b > a) s_key[lds_slot<IPT>(a - base)] = r;
      else y[r] = T(0);
    }
    __syncthreads();
  }

  // phase 2
  T acc = 0, lead = 0;
  int has_head = 0, last_key = -1, first_close_key = -1;
  bool head_at_chunk_start = false;
  int32_t kprev = prev_key;
  if (!CSR && tid > 0) kprev = s_key[lds_slot<IPT>(tid * IPT - 1)];
#pragma unroll
  for (int k = 0; k < IPT; ++k) {
    const int e = tid * IPT + k;
    const int32_t key = s_key[lds_slot<IPT>(e)];
    const T v = s_val[lds_slot<IPT>(e)];
    const bool head = CSR ? (key >= 0) : (key != kprev);
    if (head) {
      if (!has_head) {
        lead = acc;
        has_head = 1;
        first_close_key = kprev;  // COO; CSR takes it from the scan
        head_at_chunk_start = (e == 0);
      } else {
        y[CSR ? last_key : kprev] = acc;
      }
      acc = 0;
      last_key = key;
    }
    acc += v;
    if (!CSR) kprev = key;
  }

  SegSum<T> in = block_seg_exclusive_scan<T>(SegSum<T>{has_head, acc, last_key}, s_scan);

  if (has_head) {
    const T total = in.v + lead;
    if (in.f) {
      y[CSR ? in.k : first_close_key] = total;
    } else {  // first head of the chunk: what precedes it continues an earlier chunk
      carry_key[chunk] = head_at_chunk_start ? -1 : (CSR ? carry_row : first_close_key);
      carry_val[chunk] = total;
    }
  }
  if (tid == kBlock - 1) {  // the segment still open at the end of the chunk
    if (has_head) {
      y[last_key] = acc;  // COO: last_key == kprev
    } else if (in.f) {
      y[CSR ? in.k : kprev] = in.v + acc;
    } else {  // no head in the whole chunk: everything is carry
      carry_key[chunk] = CSR ? carry_row : kprev;
      carry_val[chunk] = in.v + acc;
    }
  }
}

// ---------------------------------------------------------------- CSR, short rows, streamed
// A workgroup owns 256 consecutive rows. Their entries are one contiguous range of crd /
// vals, which the lanes read side by side with 16-byte loads (no lane waits on pos to find
// its entries), multiply by x and park in LDS in pieces of kStreamCap products; then one
// lane per row adds, in order, the part of its row that lies in the piece (eight LDS reads
// per round trip). A row part longer than kStreamCoop products is added up by the whole wave
// instead (strided partial sums, then a butterfly), so one long row costs its length / 64,
// not its length. Any row length is handled; the kernel is chosen for short mean rows because
// there a piece holds many whole rows and nothing has to be searched. Fixed order of
// additions: bit-reproducible.
// Measured and left out (banded matrix, 6 entries per row, fp64, 41 us): 2 or 4 rows per lane
// (43 / 46 us: fewer, longer workgroups leave the last round of workgroups half empty);
// workgroups that stay resident and walk through their blocks with the next piece's loads
// issued before the current piece is reduced (43-45 us with 1024 or 2048 products per piece,
// at 5, 6 or 8 waves per SIMD). The kernel runs at the rate at which the memory system serves
// this mix of three streams and a gather of 64-byte pieces of x, not at a latency limit.
constexpr int kStreamRows = kBlock;  // rows per workgroup, one per lane
constexpr int kStreamCap = 2048;     // products parked per piece
constexpr int kStreamCoop = 48;      // longer row parts are summed by the whole wave
constexpr int kStreamLong = 3 * kStreamCap;  // rows from this length on take the register path

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

template <typename T, bool VEC, class XP>
__global__ __launch_bounds__(kBlock) void csr_stream_kernel(int nrows, int nnz,
                                                            const int32_t* __restrict__ pos,
                                                            const int32_t* __restrict__ crd,
                                                            const T* __restrict__ vals, const XP x,
                                                            T* __restrict__ y,
                                                            const int32_t* __restrict__ select, int want) {
  typedef int32_t i4 __attribute__((ext_vector_type(4)));
  using V = typename VecOf<T>::type;  // 16 bytes of values
  constexpr int R = VecOf<T>::R;
  if (!selected(select, want)) return;  // the other CSR kernel was chosen on the device
  __shared__ int32_t s_pos[kStreamRows + 1];
  __shared__ T s_prod[kStreamCap];
  __shared__ T s_wpart[kBlock / kWave];
  __shared__ int s_lend;
  const int tid = threadIdx.x;
  const int row0 = xcd_contiguous_block_id() * kStreamRows;
  for (int q = tid; q <= kStreamRows; q += kBlock) s_pos[q] = pos[min(row0 + q, nrows)];
  __syncthreads();
  const int e0 = s_pos[0], e1 = s_pos[kStreamRows];
  const int e0a = e0 & ~3;  // pieces start on a multiple of 4 entries: aligned 16-byte loads
  const int ra = s_pos[tid], rb = s_pos[tid + 1];
  T acc = T(0);
  // can this block hold a row of kStreamLong entries or more? (uniform; rare)
  const bool has_long = e1 - e0 >= kStreamLong;
  if (has_long) {
    if (tid == 0) s_lend = 0;
    __syncthreads();
  }
  constexpr int G = kStreamCap / (4 * kBlock);
  for (int c0 = e0a; c0 < e1; c0 += kStreamCap) {
    if (has_long) {
      // Long stretch of one row ahead: its whole pieces are added up in registers, without
      // LDS and without a barrier per piece (so the loads of consecutive pieces overlap), and
      // folded into the row's lane once. Keeps a block with a 100 000-entry row from taking
      // fifty serial load -> park -> add rounds.
      const bool mine = ra <= c0 && rb - c0 >= 2 * kStreamCap;  // at most one lane
      if (mine) s_lend = rb;
      __syncthreads();
      const int lend = s_lend;
      __syncthreads();
      if (mine) s_lend = 0;
      if (lend) {
        T part = T(0);
        int c = c0;
#pragma unroll 1
        for (; c + kStreamCap <= lend; c += kStreamCap) {
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const int p = c + 4 * (g * kBlock + tid);
            if (VEC) {
              const i4 cc = ld_stream(reinterpret_cast<const i4*>(crd + p));
              T v[4];
#pragma unroll
              for (int h = 0; h < 4 / R; ++h) {
                const V w = ld_stream(reinterpret_cast<const V*>(vals + p + R * h));
#pragma unroll
                for (int r = 0; r < R; ++r) v[R * h + r] = w[r];
              }
#pragma unroll
              for (int r = 0; r < 4; ++r) part += v[r] * x.at(cc[r]);
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) part += ld_stream(vals + p + r) * x.at(ld_stream(crd + p + r));
            }
          }
        }
        part = wave_sum(part);
        if (lane_id() == 0) s_wpart[wave_id()] = part;
        __syncthreads();
        if (mine) {
#pragma unroll
          for (int w = 0; w < kBlock / kWave; ++w) acc += s_wpart[w];
        }
        __syncthreads();
        c0 = c - kStreamCap;  // the loop's increment moves on to c
        continue;
      }
    }
    const int c1 = min(c0 + kStreamCap, e1);
    // a lane holds up to G groups of 4 consecutive entries; all their loads are issued before
    // the first use, none behind a per-lane branch: a lane without work in this piece re-reads
    // the piece's first group (one cache line for all such lanes) and parks products nobody adds
    const bool whole = VEC && c1 + 3 <= nnz;  // uniform: every 16-byte group lies inside the arrays
    T pr[G][4];
    if (whole) {
      i4 c[G];
      T v[G][4];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int p = c0 + 4 * (g * kBlock + tid);
        const int pc = p < c1 ? p : c0;
        c[g] = ld_stream(reinterpret_cast<const i4*>(crd + pc));
#pragma unroll
        for (int h = 0; h < 4 / R; ++h) {
          const V w = ld_stream(reinterpret_cast<const V*>(vals + pc + R * h));
#pragma unroll
          for (int r = 0; r < R; ++r) v[g][R * h + r] = w[r];
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) pr[g][r] = v[g][r] * x.at(c[g][r]);
    } else {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int p = c0 + 4 * (g * kBlock + tid);
#pragma unroll
        for (int r = 0; r < 4; ++r)
          pr[g][r] = p + r < c1 ? ld_stream(vals + p + r) * x.at(ld_stream(crd + p + r)) : T(0);
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int r = 0; r < 4; ++r) s_prod[4 * (g * kBlock + tid) + r] = pr[g][r];
    __syncthreads();
    const int a = max(ra, c0), e = min(rb, c1);
    const bool big = e - a > kStreamCoop;
    if (!big && a < e) {
      for (int q0 = a; q0 < e; q0 += 8) {  // reads at a clamped index, added in order
        T t[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) t[k] = s_prod[min(q0 + k, e - 1) - c0];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc += q0 + k < e ? t[k] : T(0);
      }
    }
    uint64_t todo = __ballot(big);
    while (todo) {  // uniform: the wave adds up one long row part at a time
      const int src = __ffsll(static_cast<long long>(todo)) - 1;
      todo &= todo - 1;
      const int la = __shfl(a, src), lb = __shfl(e, src);
      T part = T(0);
      for (int q = la + lane_id(); q < lb; q += kWave) part += s_prod[q - c0];
      part = wave_sum(part);
      if (lane_id() == src) acc += part;
    }
    __syncthreads();
  }
  const int r = row0 + tid;
  if (r < nrows) y[r] = acc;
}

template <typename T, class XP>
static spt_status launch_csr_stream(int64_t nnz, int64_t nrows, const int32_t* pos,
                                    const int32_t* crd, const T* vals, const XP x, T* y,
                                    hipStream_t s, const int32_t* select = nullptr, int want = 0) {
  const unsigned grid = (unsigned)((nrows + kStreamRows - 1) / kStreamRows);
  const bool vec = ((reinterpret_cast<uintptr_t>(crd) | reinterpret_cast<uintptr_t>(vals)) & 15) == 0;
  if (vec)
    hipLaunchKernelGGL((csr_stream_kernel<T, true, XP>), dim3(grid), dim3(kBlock), 0, s, (int)nrows,
                       (int)nnz, pos, crd, vals, x, y, select, want);
  else
    hipLaunchKernelGGL((csr_stream_kernel<T, false, XP>), dim3(grid), dim3(kBlock), 0, s, (int)nrows,
                       (int)nnz, pos, crd, vals, x, y, select, want);
  SPT_CHECK_LAUNCH("csr_stream");
  return SPT_OK;
}

// Which CSR kernel runs. The streamed kernel needs no search and no second launch and wins
// where rows are short (banded matrix, 6 entries per row, fp64: 42 vs 65 us; rows of 8..32
// entries, fp32: 117 vs 135 us); the entry-balanced kernel does not care how the entries are
// spread over the rows (power-law rows, mean 15, longest 10^5: 0.97 ms against 1.08 ms
// streamed). The host knows the mean row length (nvals / rows) and nothing about the spread,
// so the mean decides, and a declared bound on the longest row (max_children of the column
// level, 0 = unknown) overrides it either way.
constexpr int kStreamMeanRow = 32;
static bool csr_use_stream(int64_t nnz, int64_t nrows, int hint) {
  if (nnz < 1 || nnz >= INT32_MAX || nrows + kBlock >= INT32_MAX) return false;
  static const char* force = getenv("SPT_CSR_KERNEL");  // measurement aid: "stream" or "balanced"
  if (force && force[0] == 's') return true;
  if (force && force[0] == 'b') return false;
  if (hint > 0) return hint <= kStreamMeanRow;
  return nnz <= kStreamMeanRow * nrows;
}

// ---------------------------------------------------------------- unsorted COO
// The fused single loop over all entries of the paper's COO kernel: a scatter
// into y (Section 4.5, fusing iterators), one atomic add per entry.
template <typename T>
__global__ __launch_bounds__(kBlock) void coo_atomic_spmv_kernel(
    int nnz, const int32_t* __restrict__ row, const int32_t* __restrict__ col,
    const T* __restrict__ vals, const T* __restrict__ x, T* __restrict__ y) {
  const int p = blockIdx.x * kBlock + threadIdx.x;
  if (p >= nnz) return;
  const T prod = ld_stream(vals + p) * x[ld_stream(col + p)];
  unsafeAtomicAdd(y + ld_stream(row + p), prod);
}

// ---------------------------------------------------------------- sorted COO, small
// The whole product in one launch, for matrices whose run time is the launches themselves.
// One wave per 256 consecutive entries (four per lane). The wave that holds a row's first
// entry owns the row: it adds up the row's entries of its own piece with a segmented sum over
// the lanes and, if the row is still open at the end of the piece, keeps reading the entries
// that follow, 64 at a time, until the row changes; entries before a piece's first row start
// belong to an earlier owner and are skipped. Rows without entries lie between the rows of
// two neighbouring entries (or before the first / after the last entry) and are zeroed by the
// thread that sees the gap. No workspace, no atomics, a fixed order of additions.
constexpr int kSmallPiece = 4 * kWave;
constexpr int64_t kSmallCooMaxEntries = 1 << 16;  // worst case (one row holds everything): 1024 read-ahead rounds
constexpr int64_t kSmallCooMaxRows = 1 << 20;     // worst case (all rows empty but one): one wave zeroes them, 16 384 rounds

template <typename T>
__device__ __forceinline__ void zero_rows(T* __restrict__ y, int lo, int hi) {  // rows lo .. hi - 1
  const bool big = hi - lo > 16;
  if (!big)
    for (int r = lo; r < hi; ++r) y[r] = T(0);
  uint64_t todo = __ballot(big);
  while (todo) {  // a long run of empty rows is zeroed by the whole wave
    const int src = __ffsll(static_cast<long long>(todo)) - 1;
    todo &= todo - 1;
    const int l = __shfl(lo, src), h = __shfl(hi, src);
    for (int r = l + lane_id(); r < h; r += kWave) y[r] = T(0);
  }
}

template <typename T>
__global__ __launch_bounds__(kWave) void coo_small_spmv_kernel(int nnz, int nrows, const int32_t* __restrict__ row,
                                                               const int32_t* __restrict__ col,
                                                               const T* __restrict__ vals, const T* __restrict__ x,
                                                               T* __restrict__ y) {
  const int lane = lane_id();
  const int base = blockIdx.x * kSmallPiece;
  const int end = min(base + kSmallPiece, nnz);
  const int p0 = base + lane * 4;
  int32_t r[4], c[4];
  T v[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const bool ok = p0 + q < nnz;
    const int p = ok ? p0 + q : nnz - 1;  // beyond the end: the last entry's row again, value 0
    r[q] = row[p];
    c[q] = col[p];
    v[q] = ok ? vals[p] : T(0);
  }
  // the 64 entries after the piece, one per lane: where an open row usually ends
  const int pa = end + lane;
  const bool ahead_ok = pa < nnz;
  int32_t ra = ahead_ok ? row[pa] : -1, ca = ahead_ok ? col[pa] : 0;
  T va = ahead_ok ? vals[pa] : T(0);
  int32_t prev = dpp_move<0x138, 0xf>(-1, r[3]);  // wave_shr:1
  if (lane == 0) prev = base > 0 ? row[base - 1] : -1;
  T prod[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) prod[q] = p0 + q < nnz ? v[q] * x[c[q]] : T(0);
  const T prod_a = ahead_ok ? va * x[ca] : T(0);

  unsigned headmask = 0;
  {
    int32_t a = prev;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bool valid = p0 + q < nnz;
      if (valid && r[q] != a) headmask |= 1u << q;
      zero_rows<T>(y, valid && r[q] != a ? a + 1 : 0, valid && r[q] != a ? r[q] : 0);
      if (valid) a = r[q];
    }
    // rows after the last entry of the matrix
    const bool last_entry = p0 <= nnz - 1 && nnz - 1 < p0 + 4;
    zero_rows<T>(y, last_entry ? row[nnz - 1] + 1 : 0, last_entry ? nrows : 0);
  }

  T acc = 0;
  int has_head = 0, last_key = -1;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (headmask & (1u << q)) {
      if (has_head) y[last_key] = acc;  // a row that starts and ends inside this lane
      has_head = 1;
      last_key = r[q];
      acc = 0;
    }
    acc += prod[q];
  }
  SegSum<T> me{has_head, acc, last_key};
  wave_seg_step<0x111, 0xf>(me);
  wave_seg_step<0x112, 0xf>(me);
  wave_seg_step<0x114, 0xf>(me);
  wave_seg_step<0x118, 0xf>(me);
  wave_seg_step<0x142, 0xa>(me);
  wave_seg_step<0x143, 0xc>(me);
  SegSum<T> ex;  // what the lanes before this one add up to
  ex.f = dpp_move<0x138, 0xf>(0, me.f);
  ex.v = dpp_move<0x138, 0xf>(T(0), me.v);
  ex.k = dpp_move<0x138, 0xf>(-1, me.k);
  // the first head of a lane closes the row that was open in the lanes before it; if no lane
  // before holds a head, that row began in an earlier piece and its owner adds these entries
  if (has_head && ex.f) {
    T lead = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (headmask & (1u << q)) break;
      lead += prod[q];
    }
    y[ex.k] = ex.v + lead;
  }
  // the row still open at the end of the piece (inclusive summary of the last lane)
  const int open_f = __shfl(me.f, kWave - 1);
  if (!open_f) return;  // no row starts in this piece
  const int open_row = __shfl(me.k, kWave - 1);
  T sum = __shfl(me.v, kWave - 1);
  bool more = true;
  {
    const bool match = ahead_ok && ra == open_row;
    sum += wave_total<T>(match ? prod_a : T(0));
    more = __ballot(match) == ~uint64_t(0);
  }
  for (int q0 = end + kWave; more; q0 += kWave) {  // a long row: keep reading, 64 entries a round
    const int p = q0 + lane;
    const bool match = p < nnz && row[min(p, nnz - 1)] == open_row;
    const T t = match ? vals[p] * x[col[p]] : T(0);
    sum += wave_total<T>(t);
    more = __ballot(match) == ~uint64_t(0);
  }
  if (lane == 0) y[open_row] = sum;
}

// ---------------------------------------------------------------- launchers

// binned scatter for large unordered COO (coo_bin.hip)
template <typename T>
spt_status coo_binned_spmv(int64_t nnz, int64_t nrows, const int32_t* row, const int32_t* col,
                           const T* vals, const T* x, T* y, void* ws, size_t ws_bytes,
                           hipStream_t s);
size_t coo_binned_workspace(int dtype, int64_t nnz, int64_t nrows);
constexpr int64_t kBinnedMinEntries = 1 << 15;  // below this one atomic per entry is cheaper

size_t coo_unordered_workspace(int dtype, int64_t nnz, int64_t nrows) {
  return nnz >= kBinnedMinEntries ? coo_binned_workspace(dtype, nnz, nrows) : 256;
}

constexpr int kSegIPT = 8;

size_t seg_spmv_workspace(int64_t nnz) {
  const int64_t chunk = (int64_t)kSegIPT * kBlock;
  const int64_t nwg = (nnz + chunk - 1) / chunk;
  return align_up((size_t)nwg * 4, 256) + align_up((size_t)nwg * 8, 256) + 256;
}

template <typename T>
static spt_status launch_fill(T* out, int64_t n, T v, hipStream_t s) {
  if (n <= 0) return SPT_OK;
  const int64_t grid = (n + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(fill_kernel<T>, dim3((unsigned)grid), dim3(kBlock), 0, s, out, n, v);
  SPT_CHECK_LAUNCH("fill");
  return SPT_OK;
}

template <typename T, bool CSR, class XP>
static spt_status launch_seg_x(int64_t nnz, int64_t nrows, const int32_t* pos_or_row,
                               const int32_t* col, const T* vals, const XP x, T* y, void* ws,
                               size_t ws_bytes, hipStream_t s, const int32_t* select = nullptr,
                               int want = 0) {
  constexpr int CHUNK = kSegIPT * kBlock;
  if (nnz == 0) return launch_fill<T>(y, nrows, T(0), s);
  if (nnz + CHUNK >= INT32_MAX || nrows + 1 >= INT32_MAX)
    return fail(SPT_ERR_UNSUPPORTED, "spmv: more than 2^31 entries or rows");
  const int nwg = (int)((nnz + CHUNK - 1) / CHUNK);
  if (ws_bytes < seg_spmv_workspace(nnz) || ws == nullptr)
    return fail(SPT_ERR_WORKSPACE, "spmv: workspace of %zu bytes needed, %zu given",
                seg_spmv_workspace(nnz), ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* ckey = W.take<int32_t>(nwg);
  T* cval = W.take<T>(nwg);
  if (!CSR) {
    spt_status st = launch_fill<T>(y, nrows, T(0), s);
    if (st != SPT_OK) return st;
  }
  const bool vec = aligned16(col) && aligned16(vals) && (CSR || aligned16(pos_or_row));
  if (vec)
    hipLaunchKernelGGL((seg_spmv_kernel<T, CSR, kSegIPT, true, XP>), dim3(nwg), dim3(kBlock), 0, s,
                       (int)nnz, (int)nrows, pos_or_row, col, vals, x, y, ckey, cval, select, want);
  else
    hipLaunchKernelGGL((seg_spmv_kernel<T, CSR, kSegIPT, false, XP>), dim3(nwg), dim3(kBlock), 0, s,
                       (int)nnz, (int)nrows, pos_or_row, col, vals, x, y, ckey, cval, select, want);
  SPT_CHECK_LAUNCH("seg_spmv");
  hipLaunchKernelGGL(carry_fixup_kernel<T>, dim3((nwg + kBlock - 1) / kBlock), dim3(kBlock), 0, s,
                     nwg, ckey, cval, y, select, want);
  SPT_CHECK_LAUNCH("carry_fixup");
  return SPT_OK;
}

template <typename T, bool CSR>
static spt_status launch_seg(int64_t nnz, int64_t nrows, const int32_t* pos_or_row,
                             const int32_t* col, const T* vals, const T* x, T* y, void* ws,
                             size_t ws_bytes, hipStream_t s, const int32_t* select = nullptr,
                             int want = 0) {
  return launch_seg_x<T, CSR, DenseX<T>>(nnz, nrows, pos_or_row, col, vals, DenseX<T>{x}, y, ws,
                                         ws_bytes, s, select, want);
}

// Large CSR matrices without a declared row bound: which kernel suits is decided on the device.
// kSelectFlags workgroups look at the entry count of every block of 256 rows; if some block
// holds more than 1/kSkewShare of all entries, the streamed kernel would end on that block's
// workgroup alone (a block of 10^5 entries keeps one workgroup busy for about 0.1 ms), and the
// entry-balanced kernel runs instead. Both kernels are launched; the one not chosen returns at
// once. That costs some 10 us, which is why only matrices of kDynamicMinEntries entries or
// more (kernel times from half a millisecond) are looked at; smaller ones go by the mean alone.
constexpr int64_t kDynamicMinEntries = int64_t(1) << 25;
constexpr int kSkewShare = 1536;
__global__ __launch_bounds__(kBlock) void csr_skew_kernel(int nrows, int nnz, const int32_t* __restrict__ pos,
                                                          int32_t* __restrict__ select) {
  __shared__ int s_any;
  if (threadIdx.x == 0) s_any = 0;
  __syncthreads();
  const int nblocks = (nrows + kStreamRows - 1) / kStreamRows;
  int heavy = 0;
  for (int b = blockIdx.x * kBlock + threadIdx.x; b < nblocks; b += kSelectFlags * kBlock) {
    const int64_t e = pos[min((b + 1) * kStreamRows, nrows)] - pos[b * kStreamRows];
    heavy |= e * kSkewShare > nnz;
  }
  if (heavy) s_any = 1;
  __syncthreads();
  if (threadIdx.x == 0) select[blockIdx.x] = s_any;  // any flag set: the entry-balanced kernel
}

// y = A x, A in CSR, x a sparse vector (compressed level) or a hash map (hashed level).
template <typename T>
static spt_status spmv_sparse_x_typed(const spt_tensor* A, const spt_tensor* X, T* y, void* ws,
                                      size_t ws_bytes, hipStream_t s) {
  const spt_level& L = X->level[0];
  const T* xv = static_cast<const T*>(X->vals);
  const int64_t nnz = A->nvals, N = A->level[0].N;
  const T* vals = static_cast<const T*>(A->vals);
  if (X->nvals >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "spmv: x too large");
  const int hint = A->level[1].max_children;  // declared short rows: the streamed kernel
  const bool stream = csr_use_stream(nnz, N, hint);
  if (L.kind == SPT_HASHED) {
    if (L.M < 1) return fail(SPT_ERR_INVALID_ARG, "spmv: hashed x needs a table width W >= 1");
    if (stream)
      return launch_csr_stream<T, HashX<T>>(nnz, N, A->level[1].pos, A->level[1].crd, vals,
                                            HashX<T>{L.crd, xv, (int)L.M}, y, s);
    return launch_seg_x<T, true, HashX<T>>(nnz, N, A->level[1].pos, A->level[1].crd, vals,
                                           HashX<T>{L.crd, xv, (int)L.M}, y, ws, ws_bytes, s);
  }
  if (stream)
    return launch_csr_stream<T, SparseX<T>>(nnz, N, A->level[1].pos, A->level[1].crd, vals,
                                            SparseX<T>{L.crd, xv, (int)X->nvals}, y, s);
  return launch_seg_x<T, true, SparseX<T>>(nnz, N, A->level[1].pos, A->level[1].crd, vals,
                                           SparseX<T>{L.crd, xv, (int)X->nvals}, y, ws, ws_bytes, s);
}

spt_status spmv_sparse_x_dispatch(const spt_tensor* A, const spt_tensor* X, void* y, void* ws,
                                  size_t ws_bytes, hipStream_t s) {
  if (A->dtype == SPT_F64)
    return spmv_sparse_x_typed<double>(A, X, static_cast<double*>(y), ws, ws_bytes, s);
  return spmv_sparse_x_typed<float>(A, X, static_cast<float*>(y), ws, ws_bytes, s);
}

// y[row[r]] = t[r] for the stored rows of a doubly compressed matrix
template <typename T>
__global__ __launch_bounds__(kBlock) void scatter_rows_kernel(int n, const int32_t* __restrict__ row,
                                                              const T* __restrict__ t,
                                                              T* __restrict__ y) {
  const int r = blockIdx.x * kBlock + threadIdx.x;
  if (r < n) y[row[r]] = t[r];
}

spt_status launch_expand_parents(int n, int nparents, const int32_t* pos, int32_t* out, hipStream_t s);

size_t csc_spmv_workspace(const spt_tensor* A) {
  return align_up(static_cast<size_t>(A->nvals) * 4, 256) +
         coo_unordered_workspace(A->dtype, A->nvals, A->level[1].N);
}

size_t dcsr_spmv_workspace(const spt_tensor* A) {
  return align_up(static_cast<size_t>(A->level[1].M) * 8, 256) + seg_spmv_workspace(A->nvals);
}

template <typename T>
static spt_status spmv_typed(Format f, const spt_tensor* A, const T* x, T* y, void* ws,
                             size_t ws_bytes, hipStream_t s) {
  const T* vals = static_cast<const T*>(A->vals);
  switch (f) {
    case Format::DCSR: {
      // (compressed, compressed): the column level is a CSR over the stored rows only, so
      // the CSR kernels produce one sum per stored row, which is then placed at the row's
      // coordinate in the zero-filled y (row coordinates are unique: no two sums collide)
      const int64_t N = A->level[0].N, stored = A->level[1].M;
      spt_status st = launch_fill<T>(y, N, T(0), s);
      if (st != SPT_OK || stored == 0) return st;
      if (stored >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "spmv: more than 2^31 stored rows");
      if (!ws || ws_bytes < dcsr_spmv_workspace(A))
        return fail(SPT_ERR_WORKSPACE, "spmv: workspace of %zu bytes needed, %zu given",
                    dcsr_spmv_workspace(A), ws_bytes);
      Workspace W(ws, ws_bytes);
      T* t = reinterpret_cast<T*>(W.take<double>(stored));
      char* rest = static_cast<char*>(ws) + W.used;
      const int hint = A->level[1].max_children;
      if (csr_use_stream(A->nvals, stored, hint))
        st = launch_csr_stream<T, DenseX<T>>(A->nvals, stored, A->level[1].pos, A->level[1].crd, vals,
                                             DenseX<T>{x}, t, s);
      else
        st = launch_seg<T, true>(A->nvals, stored, A->level[1].pos, A->level[1].crd, vals, x, t, rest,
                                 ws_bytes - W.used, s);
      if (st != SPT_OK) return st;
      hipLaunchKernelGGL(scatter_rows_kernel<T>, dim3(static_cast<unsigned>((stored + kBlock - 1) / kBlock)),
                         dim3(kBlock), 0, s, static_cast<int>(stored), A->level[0].crd, t, y);
      SPT_CHECK_LAUNCH("scatter rows");
      return SPT_OK;
    }
    case Format::CSR: {
      const int hint = A->level[1].max_children;
      if (csr_use_stream(A->nvals, A->level[0].N, hint)) {
        static const bool forced = getenv("SPT_CSR_KERNEL") != nullptr;
        if (hint == 0 && A->nvals >= kDynamicMinEntries && !forced) {
          if (!ws || ws_bytes < seg_spmv_workspace(A->nvals))
            return fail(SPT_ERR_WORKSPACE, "spmv: workspace of %zu bytes needed, %zu given",
                        seg_spmv_workspace(A->nvals), ws_bytes);
          // the flags live in the last 256 bytes of the workspace, behind the carries
          int32_t* select = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + seg_spmv_workspace(A->nvals) - 256);
          hipLaunchKernelGGL(csr_skew_kernel, dim3(kSelectFlags), dim3(kBlock), 0, s, (int)A->level[0].N, (int)A->nvals,
                             A->level[1].pos, select);
          SPT_CHECK_LAUNCH("csr skew");
          spt_status st = launch_csr_stream<T, DenseX<T>>(A->nvals, A->level[0].N, A->level[1].pos,
                                                          A->level[1].crd, vals, DenseX<T>{x}, y, s, select, 0);
          if (st != SPT_OK) return st;
          return launch_seg<T, true>(A->nvals, A->level[0].N, A->level[1].pos, A->level[1].crd, vals, x, y,
                                     ws, ws_bytes, s, select, 1);
        }
        return launch_csr_stream<T, DenseX<T>>(A->nvals, A->level[0].N, A->level[1].pos,
                                               A->level[1].crd, vals, DenseX<T>{x}, y, s);
      }
      return launch_seg<T, true>(A->nvals, A->level[0].N, A->level[1].pos, A->level[1].crd, vals,
                                 x, y, ws, ws_bytes, s);
    }
    case Format::CSC: {
      // (dense columns, compressed rows): the entries lie in column order, which makes the
      // matrix a COO whose row coordinates are unordered and whose column coordinates are
      // implicit in pos. The columns are written out once, then the entries are binned by row
      // like any unordered COO; x is read in ascending order on the way.
      const int64_t nnz = A->nvals, N = A->level[1].N, M = A->level[0].N;
      if (nnz >= INT32_MAX || M + 1 >= INT32_MAX)
        return fail(SPT_ERR_UNSUPPORTED, "spmv: more than 2^31 entries or columns");
      if (nnz == 0) return launch_fill<T>(y, N, T(0), s);
      if (!ws || ws_bytes < csc_spmv_workspace(A))
        return fail(SPT_ERR_WORKSPACE, "spmv: workspace of %zu bytes needed, %zu given",
                    csc_spmv_workspace(A), ws_bytes);
      Workspace W(ws, ws_bytes);
      int32_t* cols = W.take<int32_t>(nnz);
      spt_status st = launch_expand_parents((int)nnz, (int)M, A->level[1].pos, cols, s);
      if (st != SPT_OK) return st;
      if (nnz >= kBinnedMinEntries)
        return coo_binned_spmv<T>(nnz, N, A->level[1].crd, cols, vals, x, y,
                                  static_cast<char*>(ws) + W.used, ws_bytes - W.used, s);
      st = launch_fill<T>(y, N, T(0), s);
      if (st != SPT_OK) return st;
      hipLaunchKernelGGL(coo_atomic_spmv_kernel<T>, dim3((unsigned)((nnz + kBlock - 1) / kBlock)),
                         dim3(kBlock), 0, s, (int)nnz, A->level[1].crd, cols, vals, x, y);
      SPT_CHECK_LAUNCH("coo_atomic_spmv");
      return SPT_OK;
    }
    case Format::COO2: {
      const int64_t nnz = A->nvals, N = A->level[0].N;
      if ((A->level[0].flags & SPT_ORDERED) && nnz > 0 && nnz <= kSmallCooMaxEntries && N <= kSmallCooMaxRows) {
        hipLaunchKernelGGL(coo_small_spmv_kernel<T>, dim3((unsigned)((nnz + kSmallPiece - 1) / kSmallPiece)),
                           dim3(kWave), 0, s, (int)nnz, (int)N, A->level[0].crd, A->level[1].crd, vals, x, y);
        SPT_CHECK_LAUNCH("coo_small_spmv");
        return SPT_OK;
      }
      if (A->level[0].flags & SPT_ORDERED)
        return launch_seg<T, false>(nnz, N, A->level[0].crd, A->level[1].crd, vals, x, y, ws,
                                    ws_bytes, s);
      if (nnz >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "spmv: more than 2^31 entries");
      if (nnz >= kBinnedMinEntries)
        return coo_binned_spmv<T>(nnz, N, A->level[0].crd, A->level[1].crd, vals, x, y, ws, ws_bytes,
                                  s);
      spt_status st = launch_fill<T>(y, N, T(0), s);
      if (st != SPT_OK || nnz == 0) return st;
      hipLaunchKernelGGL(coo_atomic_spmv_kernel<T>, dim3((unsigned)((nnz + kBlock - 1) / kBlock)),
                         dim3(kBlock), 0, s, (int)nnz, A->level[0].crd, A->level[1].crd, vals, x,
                         y);
      SPT_CHECK_LAUNCH("coo_atomic_spmv");
      return SPT_OK;
    }
    case Format::DIA: {
      const int64_t K = A->level[0].N, N = A->level[1].N, M = A->level[1].M;
      if (N == 0) return SPT_OK;
      if (K >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "spmv: too many diagonals");
      if (K == 0) return launch_fill<T>(y, N, T(0), s);
      constexpr int R = VecOf<T>::R;
      if (M == 0) return launch_fill<T>(y, N, T(0), s);
      if (N % R == 0 && aligned16(vals) && aligned16(y)) {
        const int64_t lanes = N / R;
        const dim3 grid((unsigned)((lanes + kBlock - 1) / kBlock));
        const int32_t* off = A->level[1].offset;
        const bool xvec = aligned16(x) && M % R == 0 && M >= R;
#define SPT_DIA_CASE(KT)                                                                       \
  case KT:                                                                                     \
    if (xvec)                                                                                  \
      hipLaunchKernelGGL((dia_spmv_vec_kernel<T, KT, true>), grid, dim3(kBlock), 0, s, N, M,   \
                         (int)K, off, vals, x, y);                                             \
    else                                                                                       \
      hipLaunchKernelGGL((dia_spmv_vec_kernel<T, KT, false>), grid, dim3(kBlock), 0, s, N, M,  \
                         (int)K, off, vals, x, y);                                             \
    break;
        switch (K <= 16 ? (int)K : 0) {
          SPT_DIA_CASE(1) SPT_DIA_CASE(2) SPT_DIA_CASE(3) SPT_DIA_CASE(4) SPT_DIA_CASE(5)
          SPT_DIA_CASE(6) SPT_DIA_CASE(7) SPT_DIA_CASE(8) SPT_DIA_CASE(9) SPT_DIA_CASE(10)
          SPT_DIA_CASE(11) SPT_DIA_CASE(12) SPT_DIA_CASE(13) SPT_DIA_CASE(14) SPT_DIA_CASE(15)
          SPT_DIA_CASE(16)
          default:
            hipLaunchKernelGGL((dia_spmv_vec_kernel<T, 0, false>), grid, dim3(kBlock), 0, s, N, M,
                               (int)K, off, vals, x, y);
        }
#undef SPT_DIA_CASE
      } else {
        hipLaunchKernelGGL(dia_spmv_kernel<T>, dim3((unsigned)((N + kBlock - 1) / kBlock)),
                           dim3(kBlock), 0, s, N, M, (int)K, A->level[1].offset, vals, x, y);
      }
      SPT_CHECK_LAUNCH("dia_spmv");
      return SPT_OK;
    }
    case Format::ELL: {
      const int64_t Wd = A->level[0].N, N = A->level[1].N;
      if (N == 0) return SPT_OK;
      if (Wd >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "spmv: ELL width too large");
      constexpr int R = VecOf<T>::R;
      if (Wd == 0 || A->level[2].N == 0) return launch_fill<T>(y, N, T(0), s);
      if (N % R == 0 && aligned16(vals) && aligned16(y) && aligned16(A->level[2].crd)) {
        const int64_t lanes = N / R;
        hipLaunchKernelGGL(ell_spmv_vec_kernel<T>, dim3((unsigned)((lanes + kBlock - 1) / kBlock)),
                           dim3(kBlock), 0, s, N, (int)Wd, A->level[2].crd, vals, x, y);
      } else {
        hipLaunchKernelGGL(ell_spmv_kernel<T>, dim3((unsigned)((N + kBlock - 1) / kBlock)),
                           dim3(kBlock), 0, s, N, (int)Wd, A->level[2].crd, vals, x, y);
      }
      SPT_CHECK_LAUNCH("ell_spmv");
      return SPT_OK;
    }
    default:
      return fail(SPT_ERR_UNSUPPORTED, "spmv: the tensor is not a CSR, COO, DIA or ELL matrix");
  }
}

// out[r] = sum over p in [pos[r], pos[r+1]) of vals[p] * x[crd[p]]: CSR SpMV, and
// equally TTV on the bottom level of a CSF tensor (rows = fibers).
spt_status csr_rows_reduce(int dtype, int64_t nnz, int64_t nrows, const int32_t* pos,
                           const int32_t* crd, const void* vals, const void* x, void* out,
                           void* ws, size_t ws_bytes, hipStream_t s) {
  // always the entry-balanced kernel: fibre lengths of a skewed tensor are far from their mean
  // (the head slices hold fibres of hundreds of entries, the rest single entries: 0.37 ms
  // against 1.24 ms with the streamed kernel on 50M entries in 8.1M fibres)
  if (dtype == SPT_F64)
    return launch_seg<double, true>(nnz, nrows, pos, crd, static_cast<const double*>(vals),
                                    static_cast<const double*>(x), static_cast<double*>(out), ws,
                                    ws_bytes, s);
  return launch_seg<float, true>(nnz, nrows, pos, crd, static_cast<const float*>(vals),
                                 static_cast<const float*>(x), static_cast<float*>(out), ws, ws_bytes,
                                 s);
}

// ---- array-of-structs COO (Section 5.2): (row, col) pairs in one array ----

__global__ __launch_bounds__(kBlock) void split_pairs_kernel(int64_t n, const int32_t* __restrict__ rc,
                                                             int32_t* __restrict__ row,
                                                             int32_t* __restrict__ col) {
  const int64_t p = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (p >= n) return;
  row[p] = rc[2 * p];  // the two loads of a lane share 8 bytes, a wave reads 512 contiguous bytes
  col[p] = rc[2 * p + 1];
}

static size_t coo_matrix_spmv_workspace(const spt_tensor* A) {
  return (A->level[0].flags & SPT_ORDERED) ? seg_spmv_workspace(A->nvals)
                                           : coo_unordered_workspace(A->dtype, A->nvals, A->level[0].N);
}

size_t aos_coo_spmv_workspace(const spt_tensor* A) {
  return 2 * align_up(static_cast<size_t>(A->nvals) * 4, 256) + coo_matrix_spmv_workspace(A);
}

spt_status spmv_dispatch(Format f, const spt_tensor* A, const void* x, void* y, void* ws,
                         size_t ws_bytes, hipStream_t s);

// The pairs are split into a row and a column array in the workspace (8 bytes read and 8
// written per entry), then the COO kernels run on those.
spt_status aos_coo_spmv_dispatch(const spt_tensor* A, const void* x, void* y, void* ws,
                                 size_t ws_bytes, hipStream_t s) {
  const int64_t nnz = A->nvals;
  const size_t need = aos_coo_spmv_workspace(A);
  if (nnz > 0 && (!ws || ws_bytes < need))
    return fail(SPT_ERR_WORKSPACE, "spmv: workspace of %zu bytes needed, %zu given", need, ws_bytes);
  spt_tensor S = *A;
  S.level[0].crd_stride = S.level[1].crd_stride = 1;
  size_t used = 0;
  if (nnz > 0) {
    Workspace W(ws, ws_bytes);
    int32_t* row = W.take<int32_t>(nnz);
    int32_t* col = W.take<int32_t>(nnz);
    used = W.used;
    hipLaunchKernelGGL(split_pairs_kernel, dim3(static_cast<unsigned>((nnz + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, nnz, A->level[0].crd, row, col);
    SPT_CHECK_LAUNCH("split pairs");
    S.level[0].crd = row;
    S.level[1].crd = col;
  }
  return spmv_dispatch(Format::COO2, &S, x, y, ws ? static_cast<char*>(ws) + used : nullptr,
                       ws_bytes > used ? ws_bytes - used : 0, s);
}

spt_status spmv_dispatch(Format f, const spt_tensor* A, const void* x, void* y, void* ws,
                         size_t ws_bytes, hipStream_t s) {
  if (A->dtype == SPT_F64)
    return spmv_typed<double>(f, A, static_cast<const double*>(x), static_cast<double*>(y), ws,
                              ws_bytes, s);
  return spmv_typed<float>(f, A, static_cast<const float*>(x), static_cast<float*>(y), ws,
                           ws_bytes, s);
}

}  // namespace spt
