// COO -> CSR (paper Section 5.4, Figure 14) on gfx950.
//
//   1. reorder (Section 4.3 "reordering"): a stable least-significant-digit
//      radix sort of the (row, col, value) records, 8 bits per pass, over the
//      significant bits of the column (ROW_COL order only) and then of the row.
//      Every pass is histogram -> exclusive scan -> stable scatter; the records
//      themselves travel, so no gather through a permutation is needed.
//   2. assemble pos. Table 3 prescribes, for a compressed level, per-row counts
//      (append_edges) followed by a running sum (append_finalize); on sorted rows
//      that sum is the position of the first entry of each row and is stored
//      directly at the row boundaries (see pos_from_sorted_rows_kernel).
// Everything is integer or bit-copy work: results are exact and deterministic.
#include "common.hpp"
#include "radix.hpp"
#include "rows.hpp"
#include "scan.hpp"

namespace spt {

// Stable scatter of one pass. Element order inside a tile is (wave, item, lane);
// a lane's rank among equal digits comes from a ballot-based match inside the
// wave plus per-wave running digit counters in LDS, so equal keys keep their
// input order. The tile is then sorted by digit inside LDS (one array at a time
// through the same buffer) so that consecutive lanes store to consecutive
// addresses of each digit's run: scattered single-lane stores cost one memory
// transaction each, exactly like random gathers. off[d * ntiles + tile] is the
// exclusive scan of hist.
template <typename VT>
__global__ __launch_bounds__(kBlock) void radix_scatter_kernel(
    int n, int shift, int key_is_row, int ntiles, const int32_t* __restrict__ off,
    const int32_t* __restrict__ row_in, const int32_t* __restrict__ col_in,
    const VT* __restrict__ val_in, int32_t* __restrict__ row_out, int32_t* __restrict__ col_out,
    VT* __restrict__ val_out) {
  __shared__ int s_cnt[kWaves][kRadix];
  __shared__ int s_gdelta[kRadix];
  __shared__ VT s_buf[kSortTile];
  int32_t* s_buf32 = reinterpret_cast<int32_t*>(s_buf);
  const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
  // neighbouring tiles store to neighbouring addresses of every digit's run: keep them on
  // one XCD so that partially written cache lines meet in the same L2
  const int tile = xcd_contiguous_block_id();
  for (int q = tid; q < kWaves * kRadix; q += kBlock) (&s_cnt[0][0])[q] = 0;
  __syncthreads();

  const int32_t* __restrict__ key_in = key_is_row ? row_in : col_in;
  const int32_t* __restrict__ oth_in = key_is_row ? col_in : row_in;
  int32_t* __restrict__ key_out = key_is_row ? row_out : col_out;
  int32_t* __restrict__ oth_out = key_is_row ? col_out : row_out;
  const int tile_base = tile * kSortTile;
  const int tile_n = min(kSortTile, n - tile_base);
  const int wave_base = tile_base + w * (kWave * kSortIPT);
  const uint64_t lanes_below = ((uint64_t)1 << lane) - 1;
  volatile int* cnt = s_cnt[w];

  int32_t key[kSortIPT], oth[kSortIPT];
  VT val[kSortIPT];
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {  // all loads of the tile are issued up front
    const int i = wave_base + k * kWave + lane;
    const bool valid = i < n;
    key[k] = valid ? key_in[i] : 0;
    oth[k] = valid ? oth_in[i] : 0;
    val[k] = valid ? val_in[i] : VT(0);
  }
  int lpos[kSortIPT];  // first the rank inside (wave, digit), later the slot in the sorted tile
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
  {  // thread d: where digit d starts inside the sorted tile and in global memory
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
      key_out[dst[k]] = kk;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k)
    if (wave_base + k * kWave + lane < n) s_buf32[lpos[k]] = oth[k];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {
    const int j = k * kBlock + tid;
    if (j < tile_n) oth_out[dst[k]] = s_buf32[j];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k)
    if (wave_base + k * kWave + lane < n) s_buf[lpos[k]] = val[k];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortIPT; ++k) {
    const int j = k * kBlock + tid;
    if (j < tile_n) val_out[dst[k]] = s_buf[j];
  }
}

template <typename VT>
__global__ __launch_bounds__(kBlock) void copy_entries_kernel(int n, const int32_t* __restrict__ col_in,
                                                              const VT* __restrict__ val_in,
                                                              int32_t* __restrict__ col_out,
                                                              VT* __restrict__ val_out) {
  const int p = blockIdx.x * kBlock + threadIdx.x;
  if (p < n) {
    col_out[p] = col_in[p];
    val_out[p] = val_in[p];
  }
}

__global__ __launch_bounds__(kBlock) void zero_i32_kernel(int32_t* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) out[i] = 0;
}

struct SortPlan {
  int passes_col, passes_row, ntiles;
  size_t rec_bytes, hist_bytes, scan_bytes, total;
};

static SortPlan plan(const spt_tensor* A, int32_t order) {
  SortPlan P;
  const int64_t nnz = A->nvals;
  const size_t vsz = A->dtype == SPT_F64 ? 8 : 4;
  P.passes_col = order == SPT_ORDER_ROW_COL ? (bits_for(A->level[1].N) + kRadixBits - 1) / kRadixBits : 0;
  P.passes_row = (bits_for(A->level[0].N) + kRadixBits - 1) / kRadixBits;
  P.ntiles = (int)((nnz + kSortTile - 1) / kSortTile);
  P.rec_bytes = align_up((size_t)nnz * 4, 256) * 2 + align_up((size_t)nnz * vsz, 256);
  P.hist_bytes = align_up((size_t)kRadix * P.ntiles * 4, 256);
  const int64_t scan_n = std::max<int64_t>((int64_t)kRadix * P.ntiles, A->level[0].N + 1);
  P.scan_bytes = scan_workspace(scan_n);
  P.total = 2 * P.rec_bytes + P.hist_bytes + P.scan_bytes + 256;
  return P;
}

size_t coo_to_csr_workspace(const spt_tensor* A) {
  return std::max(plan(A, SPT_ORDER_ROW_COL).total, plan(A, SPT_ORDER_ROW_STABLE).total);
}

template <typename VT>
static spt_status convert_typed(const spt_tensor* A, int32_t order, int32_t* pos_out,
                                int32_t* crd_out, VT* vals_out, void* ws, size_t ws_bytes,
                                hipStream_t s) {
  const int64_t nnz64 = A->nvals, N = A->level[0].N;
  if (nnz64 + kSortTile >= INT32_MAX || N + 1 >= INT32_MAX)
    return fail(SPT_ERR_UNSUPPORTED, "coo_to_csr: more than 2^31 entries or rows");
  const int nnz = (int)nnz64;
  const SortPlan P = plan(A, order);
  if (!ws || ws_bytes < P.total)
    return fail(SPT_ERR_WORKSPACE, "coo_to_csr: workspace of %zu bytes needed, %zu given", P.total,
                ws_bytes);
  const int32_t* row = A->level[0].crd;
  const int32_t* col = A->level[1].crd;
  const VT* vals = static_cast<const VT*>(A->vals);

  if (nnz == 0) {
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((N + 1 + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, pos_out, N + 1);
    SPT_CHECK_LAUNCH("zero pos");
    return SPT_OK;
  }

  Workspace W(ws, ws_bytes);
  int32_t* srow[2];
  int32_t* scol[2];
  VT* sval[2];
  for (int b = 0; b < 2; ++b) {
    srow[b] = W.take<int32_t>(nnz);
    scol[b] = W.take<int32_t>(nnz);
    sval[b] = W.take<VT>(nnz);
  }
  int32_t* hist = W.take<int32_t>((size_t)kRadix * P.ntiles);
  int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(P.scan_bytes));

  const bool sorted_in = (A->level[0].flags & SPT_ORDERED) &&
                         (order == SPT_ORDER_ROW_STABLE || (A->level[1].flags & SPT_ORDERED));
  const int32_t* sorted_rows = row;
  const unsigned egrid = (unsigned)((nnz + kBlock - 1) / kBlock);
  if (sorted_in) {
    hipLaunchKernelGGL(copy_entries_kernel<VT>, dim3(egrid), dim3(kBlock), 0, s, nnz, col, vals,
                       crd_out, vals_out);
    SPT_CHECK_LAUNCH("copy_entries");
  } else {
    const int npass = P.passes_col + P.passes_row;
    const int32_t *rin = row, *cin = col;
    const VT* vin = vals;
    for (int i = 0; i < npass; ++i) {
      const bool is_row = i >= P.passes_col;
      const int shift = kRadixBits * (is_row ? i - P.passes_col : i);
      const bool last = i == npass - 1;
      int32_t* rout = srow[i & 1];
      int32_t* cout = last ? crd_out : scol[i & 1];
      VT* vout = last ? vals_out : sval[i & 1];
      spt_status hs = launch_radix_hist(is_row ? rin : cin, nnz, shift, P.ntiles, hist, s);
      if (hs != SPT_OK) return hs;
      spt_status st = device_scan_i32<false>(hist, hist, (int64_t)kRadix * P.ntiles, scan_tmp, s);
      if (st != SPT_OK) return st;
      hipLaunchKernelGGL(radix_scatter_kernel<VT>, dim3(P.ntiles), dim3(kBlock), 0, s, nnz, shift,
                         (int)is_row, P.ntiles, hist, rin, cin, vin, rout, cout, vout);
      SPT_CHECK_LAUNCH("radix_scatter");
      rin = rout;
      cin = cout;
      vin = vout;
    }
    sorted_rows = rin;
  }
  spt_status ps = launch_pos_from_sorted_rows(sorted_rows, nnz, (int)N, pos_out, s);
  if (ps != SPT_OK) return ps;
  return SPT_OK;
}

spt_status coo_to_csr_dispatch(const spt_tensor* A, int32_t order, int32_t* pos_out,
                               int32_t* crd_out, void* vals_out, void* ws, size_t ws_bytes,
                               hipStream_t s) {
  if (A->dtype == SPT_F64)
    return convert_typed<uint64_t>(A, order, pos_out, crd_out, static_cast<uint64_t*>(vals_out), ws,
                                   ws_bytes, s);
  return convert_typed<uint32_t>(A, order, pos_out, crd_out, static_cast<uint32_t*>(vals_out), ws,
                                 ws_bytes, s);
}

}  // namespace spt
