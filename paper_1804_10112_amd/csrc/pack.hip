// Packing ordered COO into other formats (Section 3.4: a result is assembled level by level
// through appends and inserts), gfx950:
//   COO3 -> CSF   three compressed levels; a coordinate is appended to level 0 / 1 where
//                 (i) / (i,j) changes, pos of a level holds where its parent's segment starts
//   COO/CSR -> ELL  cell (k, i) = k-th entry of row i, padding marked by column -1
//   COO -> DIA    the distinct offsets col - row, then one value array per diagonal
// All index work is exact and deterministic; values are copied bit for bit.
#include "common.hpp"
#include "rows.hpp"
#include "scan.hpp"

namespace spt {

__global__ __launch_bounds__(kBlock) void fill_i32_kernel(int32_t* __restrict__ out, int64_t n,
                                                          int32_t v) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < n) out[i] = v;
}

template <typename VT>
__global__ __launch_bounds__(kBlock) void fill_vt_kernel(VT* __restrict__ out, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < n) out[i] = VT(0);
}

// ================================================================ COO3 -> CSF

constexpr int kPkIPT = 8;
constexpr int kPkChunk = kPkIPT * kBlock;

// Loads a lane's kPkIPT consecutive (i, j) and marks where (i) and (i,j) change.
struct HeadMasks {
  unsigned slice, fiber;
};
template <bool VEC>
__device__ __forceinline__ HeadMasks load_heads(int nnz, int p0, const int32_t* __restrict__ ci,
                                                const int32_t* __restrict__ cj, int32_t* li,
                                                int32_t* lj) {
  typedef int32_t i4 __attribute__((ext_vector_type(4)));
  static_assert(kPkIPT == 8, "two 16-byte loads per array and lane");
  int32_t qi = -1, qj = -1;
  if (p0 > 0 && p0 < nnz) {
    qi = ci[p0 - 1];
    qj = cj[p0 - 1];
  }
  if (VEC && p0 + kPkIPT <= nnz) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const i4 a = *reinterpret_cast<const i4*>(ci + p0 + 4 * h);
      const i4 b = *reinterpret_cast<const i4*>(cj + p0 + 4 * h);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        li[4 * h + r] = a[r];
        lj[4 * h + r] = b[r];
      }
    }
  } else {
#pragma unroll
    for (int k = 0; k < kPkIPT; ++k) {
      li[k] = p0 + k < nnz ? ci[p0 + k] : -1;
      lj[k] = p0 + k < nnz ? cj[p0 + k] : -1;
    }
  }
  HeadMasks m{0, 0};
#pragma unroll
  for (int k = 0; k < kPkIPT; ++k) {
    if (p0 + k < nnz) {
      const bool s = li[k] != qi;  // the first entry differs from (-1, -1)
      if (s) m.slice |= 1u << k;
      if (s || lj[k] != qj) m.fiber |= 1u << k;
    }
    qi = li[k];
    qj = lj[k];
  }
  return m;
}

// heads0[w], heads1[w] = slices / fibres that start inside chunk w.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void csf_count_kernel(int nnz, const int32_t* __restrict__ ci,
                                                           const int32_t* __restrict__ cj,
                                                           int32_t* __restrict__ heads0,
                                                           int32_t* __restrict__ heads1) {
  int32_t li[kPkIPT], lj[kPkIPT];
  const HeadMasks m =
      load_heads<VEC>(nnz, blockIdx.x * kPkChunk + threadIdx.x * kPkIPT, ci, cj, li, lj);
  int t0, t1;
  block_inclusive_sum(__popc(m.slice), &t0);
  block_inclusive_sum(__popc(m.fiber), &t1);
  if (threadIdx.x == 0) {
    heads0[blockIdx.x] = t0;
    heads1[blockIdx.x] = t1;
  }
}

template <typename VT, bool VEC>
__global__ __launch_bounds__(kBlock) void csf_fill_kernel(
    int nnz, const int32_t* __restrict__ ci, const int32_t* __restrict__ cj,
    const int32_t* __restrict__ ck, const VT* __restrict__ vals, const int32_t* __restrict__ off0,
    const int32_t* __restrict__ off1, int32_t* __restrict__ crd0, int32_t* __restrict__ pos1,
    int32_t* __restrict__ crd1, int32_t* __restrict__ pos2, int32_t* __restrict__ crd2,
    VT* __restrict__ vals_out) {
  const int base = blockIdx.x * kPkChunk;
  const int p0 = base + threadIdx.x * kPkIPT;
  int32_t li[kPkIPT], lj[kPkIPT];
  const HeadMasks m = load_heads<VEC>(nnz, p0, ci, cj, li, lj);
  const int c0 = __popc(m.slice), c1 = __popc(m.fiber);
  int t;
  int run0 = off0[blockIdx.x] + block_inclusive_sum(c0, &t) - c0 - 1;
  int run1 = off1[blockIdx.x] + block_inclusive_sum(c1, &t) - c1 - 1;
#pragma unroll
  for (int k = 0; k < kPkIPT; ++k) {
    if (m.fiber & (1u << k)) {  // append (i,j)'s j to level 1; its leaves start at this entry
      ++run1;
      crd1[run1] = lj[k];
      pos2[run1] = p0 + k;
    }
    if (m.slice & (1u << k)) {  // append i to level 0; its fibres start at the one just appended
      ++run0;
      crd0[run0] = li[k];
      pos1[run0] = run1;
    }
  }
  // level 2 takes every entry: coordinates and values are copied, lanes side by side
  const int end = min(base + kPkChunk, nnz);
  for (int p = base + threadIdx.x; p < end; p += kBlock) {
    crd2[p] = ck[p];
    vals_out[p] = vals[p];
  }
}

// Closes the last segments (append_finalize) and reports the counts.
__global__ void csf_final_kernel(int nch, int nnz, const int32_t* __restrict__ heads0,
                                 const int32_t* __restrict__ off0,
                                 const int32_t* __restrict__ heads1,
                                 const int32_t* __restrict__ off1, int32_t* __restrict__ pos0,
                                 int32_t* __restrict__ pos1, int32_t* __restrict__ pos2,
                                 int64_t* __restrict__ counts) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const int nsl = nch > 0 ? off0[nch - 1] + heads0[nch - 1] : 0;
  const int nfib = nch > 0 ? off1[nch - 1] + heads1[nch - 1] : 0;
  pos0[0] = 0;
  pos0[1] = nsl;
  pos1[nsl] = nfib;
  pos2[nfib] = nnz;
  counts[0] = nsl;
  counts[1] = nfib;
}

size_t pack_csf_workspace(int64_t nnz) {
  const int64_t nch = (nnz + kPkChunk - 1) / kPkChunk;
  return 4 * align_up(static_cast<size_t>(nch + 1) * 4, 256) + scan_workspace(nch) + 256;
}

template <typename VT>
static spt_status pack_csf_typed(const spt_tensor* B, int32_t* pos0, int32_t* crd0, int32_t* pos1,
                                 int32_t* crd1, int32_t* pos2, int32_t* crd2, VT* vals_out,
                                 int64_t* counts, void* ws, size_t ws_bytes, hipStream_t s) {
  const int64_t nnz64 = B->nvals;
  if (nnz64 + kPkChunk >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "to_csf: more than 2^31 entries");
  const int nnz = static_cast<int>(nnz64);
  const int nch = (nnz + kPkChunk - 1) / kPkChunk;
  if (nch > 0 && (!ws || ws_bytes < pack_csf_workspace(nnz)))
    return fail(SPT_ERR_WORKSPACE, "to_csf: workspace of %zu bytes needed, %zu given",
                pack_csf_workspace(nnz), ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t *heads0 = nullptr, *off0 = nullptr, *heads1 = nullptr, *off1 = nullptr;
  if (nch > 0) {
    heads0 = W.take<int32_t>(nch + 1);
    off0 = W.take<int32_t>(nch + 1);
    heads1 = W.take<int32_t>(nch + 1);
    off1 = W.take<int32_t>(nch + 1);
    int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace(nch)));
    const int32_t *ci = B->level[0].crd, *cj = B->level[1].crd, *ck = B->level[2].crd;
    const VT* vals = static_cast<const VT*>(B->vals);
    const bool vec = ((reinterpret_cast<uintptr_t>(ci) | reinterpret_cast<uintptr_t>(cj)) & 15) == 0;
    if (vec)
      hipLaunchKernelGGL(csf_count_kernel<true>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, heads0,
                         heads1);
    else
      hipLaunchKernelGGL(csf_count_kernel<false>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, heads0,
                         heads1);
    SPT_CHECK_LAUNCH("csf count");
    spt_status st = device_scan_i32<false>(heads0, off0, nch, scan_tmp, s);
    if (st != SPT_OK) return st;
    st = device_scan_i32<false>(heads1, off1, nch, scan_tmp, s);
    if (st != SPT_OK) return st;
    if (vec)
      hipLaunchKernelGGL((csf_fill_kernel<VT, true>), dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, ck,
                         vals, off0, off1, crd0, pos1, crd1, pos2, crd2, vals_out);
    else
      hipLaunchKernelGGL((csf_fill_kernel<VT, false>), dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, ck,
                         vals, off0, off1, crd0, pos1, crd1, pos2, crd2, vals_out);
    SPT_CHECK_LAUNCH("csf fill");
  }
  hipLaunchKernelGGL(csf_final_kernel, dim3(1), dim3(kWave), 0, s, nch, nnz, heads0, off0, heads1, off1,
                     pos0, pos1, pos2, counts);
  SPT_CHECK_LAUNCH("csf final");
  return SPT_OK;
}

spt_status pack_csf_dispatch(const spt_tensor* B, int32_t* pos0, int32_t* crd0, int32_t* pos1,
                             int32_t* crd1, int32_t* pos2, int32_t* crd2, void* vals_out,
                             int64_t* counts, void* ws, size_t ws_bytes, hipStream_t s) {
  if (B->dtype == SPT_F64)
    return pack_csf_typed<uint64_t>(B, pos0, crd0, pos1, crd1, pos2, crd2,
                                    static_cast<uint64_t*>(vals_out), counts, ws, ws_bytes, s);
  return pack_csf_typed<uint32_t>(B, pos0, crd0, pos1, crd1, pos2, crd2,
                                  static_cast<uint32_t*>(vals_out), counts, ws, ws_bytes, s);
}

// ================================================================ COO / CSR -> ELL

__global__ void set_i32_kernel(int32_t* out, int32_t v) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *out = v;
}

// A workgroup packs 256 consecutive rows. Their entries are one contiguous range of col /
// vals: it is read lanes side by side in pieces of kEllCap entries into LDS, and every lane
// then writes its row's cells (k, row) from LDS - neighbouring lanes write neighbouring
// cells of the same slot - and the padding once the row has ended. The longest row is reduced
// per workgroup and merged with one atomic.
constexpr int kEllCap = 2048;
template <typename VT>
__global__ __launch_bounds__(kBlock) void ell_rows_kernel(int N, int W, const int32_t* __restrict__ pos,
                                                          const int32_t* __restrict__ col,
                                                          const VT* __restrict__ vals,
                                                          int32_t* __restrict__ crd_out,
                                                          VT* __restrict__ vals_out,
                                                          int32_t* __restrict__ longest) {
  __shared__ int32_t s_col[kEllCap];
  __shared__ VT s_val[kEllCap];
  __shared__ int s_range[2];
  __shared__ int s_max[kBlock / kWave];
  const int row0 = blockIdx.x * kBlock;
  const int i = row0 + threadIdx.x;
  const bool live = i < N;
  const int a = live ? pos[i] : 0;
  const int len = live ? pos[i + 1] - a : 0;
  if (threadIdx.x == 0) {
    s_range[0] = a;
    s_range[1] = pos[min(row0 + kBlock, N)];
  }
  __syncthreads();
  const int e0 = s_range[0], e1 = s_range[1];
  const int stored = min(len, W);  // slots of this row that hold entries
  for (int c0 = e0; c0 < e1; c0 += kEllCap) {
    const int c1 = min(c0 + kEllCap, e1);
    for (int q = c0 + threadIdx.x; q < c1; q += kBlock) {
      s_col[q - c0] = col[q];
      s_val[q - c0] = vals[q];
    }
    __syncthreads();
    // slots of this row whose entries lie in the piece: k in [max(c0 - a, 0), min(c1 - a, stored))
    const int k_lo = max(c0 - a, 0), k_hi = min(c1 - a, stored);
    if (live)
      for (int k = k_lo; k < k_hi; ++k) {
        crd_out[static_cast<int64_t>(k) * N + i] = s_col[a + k - c0];
        vals_out[static_cast<int64_t>(k) * N + i] = s_val[a + k - c0];
      }
    __syncthreads();
  }
  if (live)
    for (int k = stored; k < W; ++k) {
      crd_out[static_cast<int64_t>(k) * N + i] = -1;
      vals_out[static_cast<int64_t>(k) * N + i] = VT(0);
    }
  int m = len;
  for (int d = kWave / 2; d > 0; d >>= 1) m = max(m, __shfl_down(m, d, kWave));
  if (lane_id() == 0) s_max[wave_id()] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kBlock / kWave; ++w) m = max(m, s_max[w]);
    if (m > 0) atomicMax(longest, m);
  }
}

size_t pack_ell_workspace(Format f, const spt_tensor* A) {
  return f == Format::COO2 ? align_up(static_cast<size_t>(A->level[0].N + 1) * 4, 256) + 256 : 256;
}

template <typename VT>
static spt_status pack_ell_typed(Format f, const spt_tensor* A, int W, int32_t* crd_out, VT* vals_out,
                                 int32_t* longest, void* ws, size_t ws_bytes, hipStream_t s) {
  const int64_t N = A->level[0].N, nnz = A->nvals;
  if (N + 1 >= INT32_MAX || nnz >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "to_ell: matrix too large");
  hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(kWave), 0, s, longest, 0);
  SPT_CHECK_LAUNCH("ell set longest");
  if (N == 0) return SPT_OK;
  const int32_t* pos;
  const int32_t* col = A->level[1].crd;
  if (f == Format::CSR) {
    pos = A->level[1].pos;
  } else {
    if (!ws || ws_bytes < pack_ell_workspace(f, A))
      return fail(SPT_ERR_WORKSPACE, "to_ell: workspace of %zu bytes needed, %zu given",
                  pack_ell_workspace(f, A), ws_bytes);
    Workspace Wk(ws, ws_bytes);
    int32_t* p = Wk.take<int32_t>(N + 1);
    if (nnz > 0) {
      spt_status st = launch_pos_from_sorted_rows(A->level[0].crd, static_cast<int>(nnz),
                                                  static_cast<int>(N), p, s);
      if (st != SPT_OK) return st;
    } else {
      hipLaunchKernelGGL(fill_i32_kernel, dim3(static_cast<unsigned>((N + 1 + kBlock - 1) / kBlock)),
                         dim3(kBlock), 0, s, p, N + 1, 0);
      SPT_CHECK_LAUNCH("ell zero pos");
    }
    pos = p;
  }
  hipLaunchKernelGGL(ell_rows_kernel<VT>, dim3(static_cast<unsigned>((N + kBlock - 1) / kBlock)),
                     dim3(kBlock), 0, s, static_cast<int>(N), W, pos, col,
                     static_cast<const VT*>(A->vals), crd_out, vals_out, longest);
  SPT_CHECK_LAUNCH("ell rows");
  return SPT_OK;
}

// ================================================================ COO -> DIA

// flag[col - row + N - 1] = 1 for every stored entry (equal stores may race, harmlessly)
__global__ __launch_bounds__(kBlock) void dia_mark_kernel(int nnz, int N, const int32_t* __restrict__ row,
                                                          const int32_t* __restrict__ col,
                                                          int32_t* __restrict__ flag) {
  const int p = blockIdx.x * kBlock + threadIdx.x;
  if (p < nnz) flag[col[p] - row[p] + N - 1] = 1;
}

// The flagged offsets in ascending order: offset f - (N-1) lands at index idx[f].
__global__ __launch_bounds__(kBlock) void dia_collect_kernel(int64_t nflags, int N,
                                                             const int32_t* __restrict__ flag,
                                                             const int32_t* __restrict__ idx,
                                                             int32_t* __restrict__ offsets, int64_t cap,
                                                             int64_t* __restrict__ K_out) {
  const int64_t f = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (f >= nflags) return;
  if (flag[f] && idx[f] < cap) offsets[idx[f]] = static_cast<int32_t>(f - (N - 1));
  if (f == nflags - 1) *K_out = static_cast<int64_t>(idx[f]) + flag[f];
}

size_t dia_offsets_workspace(const spt_tensor* A) {
  const int64_t nflags = A->level[0].N + A->level[1].N;
  return 2 * align_up(static_cast<size_t>(nflags) * 4, 256) + scan_workspace(nflags) + 256;
}

spt_status dia_offsets_dispatch(const spt_tensor* A, int32_t* offsets_out, int64_t cap, int64_t* K_dev,
                                void* ws, size_t ws_bytes, hipStream_t s) {
  const int64_t N = A->level[0].N, M = A->level[1].N, nnz = A->nvals;
  const int64_t nflags = N + M - 1;
  if (nflags + 1 >= INT32_MAX || nnz >= INT32_MAX)
    return fail(SPT_ERR_UNSUPPORTED, "dia_offsets: matrix too large");
  if (nflags <= 0) return fail(SPT_ERR_INVALID_ARG, "dia_offsets: empty matrix shape");
  if (!ws || ws_bytes < dia_offsets_workspace(A))
    return fail(SPT_ERR_WORKSPACE, "dia_offsets: workspace of %zu bytes needed, %zu given",
                dia_offsets_workspace(A), ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* flag = W.take<int32_t>(nflags);
  int32_t* idx = W.take<int32_t>(nflags);
  int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace(nflags)));
  const unsigned fgrid = static_cast<unsigned>((nflags + kBlock - 1) / kBlock);
  hipLaunchKernelGGL(fill_i32_kernel, dim3(fgrid), dim3(kBlock), 0, s, flag, nflags, 0);
  SPT_CHECK_LAUNCH("dia zero flags");
  if (nnz > 0) {
    hipLaunchKernelGGL(dia_mark_kernel, dim3(static_cast<unsigned>((nnz + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, static_cast<int>(nnz), static_cast<int>(N), A->level[0].crd,
                       A->level[1].crd, flag);
    SPT_CHECK_LAUNCH("dia mark");
  }
  spt_status st = device_scan_i32<false>(flag, idx, nflags, scan_tmp, s);
  if (st != SPT_OK) return st;
  hipLaunchKernelGGL(dia_collect_kernel, dim3(fgrid), dim3(kBlock), 0, s, nflags, static_cast<int>(N),
                     flag, idx, offsets_out, cap, K_dev);
  SPT_CHECK_LAUNCH("dia collect");
  return SPT_OK;
}

// vals[d * N + row] = value, d = index of col - row in the ascending offsets (entries on
// other diagonals are skipped)
template <typename VT>
__global__ __launch_bounds__(kBlock) void dia_scatter_kernel(int nnz, int N, int K,
                                                             const int32_t* __restrict__ row,
                                                             const int32_t* __restrict__ col,
                                                             const VT* __restrict__ vals,
                                                             const int32_t* __restrict__ offsets,
                                                             VT* __restrict__ out) {
  const int p = blockIdx.x * kBlock + threadIdx.x;
  if (p >= nnz) return;
  const int i = row[p], o = col[p] - i;
  int lo = 0, hi = K;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (offsets[mid] < o) lo = mid + 1; else hi = mid;
  }
  if (lo < K && offsets[lo] == o) out[static_cast<int64_t>(lo) * N + i] = vals[p];
}

template <typename VT>
static spt_status pack_dia_typed(const spt_tensor* A, int K, const int32_t* offsets, VT* vals_out,
                                 hipStream_t s) {
  const int64_t N = A->level[0].N, nnz = A->nvals;
  if (N >= INT32_MAX || nnz >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "to_dia: matrix too large");
  const int64_t cells = static_cast<int64_t>(K) * N;
  if (cells > 0) {
    hipLaunchKernelGGL(fill_vt_kernel<VT>, dim3(static_cast<unsigned>((cells + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, vals_out, cells);
    SPT_CHECK_LAUNCH("dia zero values");
  }
  if (nnz > 0 && K > 0) {
    hipLaunchKernelGGL(dia_scatter_kernel<VT>, dim3(static_cast<unsigned>((nnz + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, static_cast<int>(nnz), static_cast<int>(N), K,
                       A->level[0].crd, A->level[1].crd, static_cast<const VT*>(A->vals), offsets,
                       vals_out);
    SPT_CHECK_LAUNCH("dia scatter");
  }
  return SPT_OK;
}

spt_status pack_dia_dispatch(const spt_tensor* A, int32_t K, const int32_t* offsets, void* vals_out,
                             hipStream_t s) {
  if (A->dtype == SPT_F64) return pack_dia_typed<uint64_t>(A, K, offsets, static_cast<uint64_t*>(vals_out), s);
  return pack_dia_typed<uint32_t>(A, K, offsets, static_cast<uint32_t*>(vals_out), s);
}

// ================================================================ COO -> (dense rows, hashed cols)

// Table 3's hashed insert on the device: insert_init is the fill with -1; an entry (i, j) then
// walks the probe sequence of locate (Table 2: from j % W, +1 with wrap) inside row i's segment
// and claims the first empty slot with a compare-and-swap, or finds j already there. Which of
// two colliding coordinates gets the earlier slot depends on the order the lanes arrive: the
// table is one of the valid ones, not a fixed one. Entries of a full segment are counted.
template <typename VT>
__global__ __launch_bounds__(kBlock) void hashed_insert_kernel(int nnz, int W,
                                                               const int32_t* __restrict__ row,
                                                               const int32_t* __restrict__ col,
                                                               const VT* __restrict__ vals,
                                                               int32_t* __restrict__ crd,
                                                               VT* __restrict__ out,
                                                               int32_t* __restrict__ dropped) {
  const int p = blockIdx.x * kBlock + threadIdx.x;
  if (p >= nnz) return;
  const int j = col[p];
  const int64_t base = static_cast<int64_t>(row[p]) * W;
  int q = j % W;
  for (int t = 0; t < W; ++t) {  // at most one full cycle
    const int32_t seen = atomicCAS(crd + base + q, -1, j);
    if (seen == -1 || seen == j) {
      out[base + q] = vals[p];
      return;
    }
    q = q + 1 == W ? 0 : q + 1;
  }
  atomicAdd(dropped, 1);
}

template <typename VT>
static spt_status pack_hashed_typed(const spt_tensor* A, int W, int32_t* crd_out, VT* vals_out,
                                    int32_t* dropped, hipStream_t s) {
  const int64_t N = A->level[0].N, nnz = A->nvals, cells = N * W;
  if (nnz >= INT32_MAX || N >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "to_hashed_rows: matrix too large");
  hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(kWave), 0, s, dropped, 0);
  SPT_CHECK_LAUNCH("hashed set dropped");
  if (cells > 0) {
    const unsigned g = static_cast<unsigned>((cells + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(g), dim3(kBlock), 0, s, crd_out, cells, -1);
    hipLaunchKernelGGL(fill_vt_kernel<VT>, dim3(g), dim3(kBlock), 0, s, vals_out, cells);
    SPT_CHECK_LAUNCH("hashed insert_init");
  }
  if (nnz > 0) {
    hipLaunchKernelGGL(hashed_insert_kernel<VT>, dim3(static_cast<unsigned>((nnz + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, static_cast<int>(nnz), W, A->level[0].crd, A->level[1].crd,
                       static_cast<const VT*>(A->vals), crd_out, vals_out, dropped);
    SPT_CHECK_LAUNCH("hashed insert");
  }
  return SPT_OK;
}

spt_status pack_hashed_dispatch(const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                                int32_t* dropped, hipStream_t s) {
  if (A->dtype == SPT_F64)
    return pack_hashed_typed<uint64_t>(A, W, crd_out, static_cast<uint64_t*>(vals_out), dropped, s);
  return pack_hashed_typed<uint32_t>(A, W, crd_out, static_cast<uint32_t*>(vals_out), dropped, s);
}

spt_status pack_ell_dispatch(Format f, const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                             int32_t* longest, void* ws, size_t ws_bytes, hipStream_t s) {
  if (A->dtype == SPT_F64)
    return pack_ell_typed<uint64_t>(f, A, W, crd_out, static_cast<uint64_t*>(vals_out), longest, ws,
                                    ws_bytes, s);
  return pack_ell_typed<uint32_t>(f, A, W, crd_out, static_cast<uint32_t*>(vals_out), longest, ws,
                                  ws_bytes, s);
}

}  // namespace spt
