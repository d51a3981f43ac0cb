// Sparse addition with a sparse result, A = B + C: COO + COO and CSR + CSR matrices
// (Section 5.2) and 3rd-order PLUS on COO (Section 5.3), gfx950.
//
// The result's coordinates are the union of the operands' coordinates, enumerated
// in order by the two-way merge of Section 4.4, and the result is assembled by
// appending (Section 3.4 / Table 3: coordinates are produced in order, pos of a CSR
// result is counts + running sum). The serial merge becomes:
//   1. merge_partition_kernel: where every tile of 1792 merge steps starts;
//   2. add_merge_kernel: per tile, stage both coordinate lists in LDS, every lane
//      walks 7 steps of the merge and notes which steps produce a result entry and
//      from which stored entries; the tile's notes are compacted in LDS, written to
//      the workspace, and the tile's result count is stored;
//   3. running sum of the tile counts (= where each tile appends);
//   4. add_fill_kernel: one lane per result entry copies the coordinates and adds
//      the one or two values it was noted to come from.
// Ties take the B entry first: a B entry whose twin in C follows produces nothing,
// the C entry then produces the sum. Everything is deterministic; a value is either
// copied or the single rounded sum b + c.
// CSR operands are first expanded to (row, col) lists; the result's pos is assembled
// from the ordered result rows.
#include "common.hpp"
#include "merge.hpp"
#include "rows.hpp"
#include "scan.hpp"

namespace spt {

constexpr int kAddVT = 7;
constexpr int kAddTile = kBlock * kAddVT;
constexpr uint32_t kNoSrc = 0xFFFF;

// rec = (index into the tile's C list or kNoSrc) << 16 | (1 + index into the tile's B list,
// 0 being the B entry just before the tile, or kNoSrc)
// UNION: every coordinate of B or C produces a result entry (addition); otherwise only the
// coordinates stored in both do (element-wise multiplication, the intersection merge).
template <typename KL, bool UNION>
__global__ __launch_bounds__(kBlock) void add_merge_kernel(const KL kb, const KL kc, int nb, int nc,
                                                           const int* __restrict__ xs,
                                                           uint32_t* __restrict__ rec,
                                                           int32_t* __restrict__ counts) {
  typedef typename KL::Key Key;
  // [0] the B entry before the tile, the tile's B entries, its C entries, the C entry after
  // the tile, one spare slot (the walk reads one entry ahead)
  __shared__ Key sK[kAddTile + 3];
  __shared__ uint32_t s_rec[kAddTile];

  const int tile = blockIdx.x;
  const int64_t total = static_cast<int64_t>(nb) + nc;
  const int64_t d0 = static_cast<int64_t>(tile) * kAddTile;
  const int64_t d1 = d0 + kAddTile < total ? d0 + kAddTile : total;
  const int x0 = xs[tile], x1 = xs[tile + 1];
  const int y0 = static_cast<int>(d0 - x0);
  const int nbl = x1 - x0, ncl = static_cast<int>(d1 - d0) - nbl;
  for (int q = threadIdx.x; q <= nbl; q += kBlock)
    sK[q] = (x0 + q > 0) ? kb.load(x0 + q - 1) : KL::none();
  Key* sC = sK + nbl + 1;
  for (int q = threadIdx.x; q <= ncl; q += kBlock)
    sC[q] = (y0 + q < nc) ? kc.load(y0 + q) : KL::none();
  __syncthreads();
  const Key* sB = sK + 1;

  const int span = nbl + ncl;
  const int dt = min(static_cast<int>(threadIdx.x) * kAddVT, span);
  const int dend = min(dt + kAddVT, span);
  int lo = dt > ncl ? dt - ncl : 0, hi = dt < nbl ? dt : nbl;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (key_le(sB[mid], sC[dt - 1 - mid])) lo = mid + 1; else hi = mid;
  }
  int x = lo, y = dt - lo;
  Key prev_b = sB[x - 1], head_b = sB[x], head_c = sC[y];
  constexpr uint32_t kNothing = 0xFFFFFFFFu;  // this step produces no result entry
  uint32_t mine[kAddVT];
  int cnt = 0;
#pragma unroll
  for (int k = 0; k < kAddVT; ++k) {
    mine[k] = kNothing;
    if (dt + k < dend) {
      const bool take_b = y >= ncl || (x < nbl && key_le(head_b, head_c));
      if (take_b) {
        // head_c is the next C entry, also past the tile's end: an equal one is this entry's twin
        if (UNION && !key_eq(head_b, head_c)) mine[k] = (kNoSrc << 16) | static_cast<uint32_t>(x + 1);
        prev_b = head_b;
        head_b = sB[++x];
      } else {
        const uint32_t bsrc = key_eq(prev_b, head_c) ? static_cast<uint32_t>(x) : kNoSrc;
        if (UNION || bsrc != kNoSrc) mine[k] = (static_cast<uint32_t>(y) << 16) | bsrc;
        head_c = sC[++y];
      }
      cnt += mine[k] != kNothing ? 1 : 0;
    }
  }
  int tile_cnt;
  int slot = block_inclusive_sum(cnt, &tile_cnt) - cnt;
#pragma unroll
  for (int k = 0; k < kAddVT; ++k)
    if (mine[k] != kNothing) s_rec[slot++] = mine[k];
  __syncthreads();
  uint32_t* out = rec + static_cast<int64_t>(tile) * kAddTile;
  for (int q = threadIdx.x; q < tile_cnt; q += kBlock) out[q] = s_rec[q];
  if (threadIdx.x == 0) counts[tile] = tile_cnt;
}

__global__ void add_total_kernel(int ntiles, const int32_t* __restrict__ counts,
                                 const int32_t* __restrict__ offs, int64_t* __restrict__ out_nnz) {
  if (threadIdx.x == 0 && blockIdx.x == 0)
    *out_nnz = ntiles > 0 ? static_cast<int64_t>(offs[ntiles - 1]) + counts[ntiles - 1] : 0;
}

struct CoordArrays {
  const int32_t *a0, *a1, *a2;  // a2 == nullptr for matrices
};
struct CoordOut {
  int32_t *a0, *a1, *a2;
};

template <typename T, bool UNION>
__global__ __launch_bounds__(kBlock) void add_fill_kernel(
    const int* __restrict__ xs, const uint32_t* __restrict__ rec, const int32_t* __restrict__ counts,
    const int32_t* __restrict__ offs, const CoordArrays B, const T* __restrict__ bv,
    const CoordArrays C, const T* __restrict__ cv, const CoordOut O, T* __restrict__ ov) {
  const int tile = blockIdx.x;
  const int cnt = counts[tile], off = offs[tile];
  const int x0 = xs[tile];
  const int y0 = static_cast<int>(static_cast<int64_t>(tile) * kAddTile - x0);
  const uint32_t* in = rec + static_cast<int64_t>(tile) * kAddTile;
  for (int q = threadIdx.x; q < cnt; q += kBlock) {
    const uint32_t r = in[q];
    const uint32_t bs = r & 0xFFFF, cs = r >> 16;
    T v = T(0);
    int32_t c0 = 0, c1 = 0, c2 = 0;
    if (bs != kNoSrc) {
      const int p = x0 - 1 + static_cast<int>(bs);
      v = bv[p];
      c0 = B.a0[p];
      c1 = B.a1[p];
      if (B.a2) c2 = B.a2[p];
    }
    if (cs != kNoSrc) {
      const int p = y0 + static_cast<int>(cs);
      if (UNION) v += cv[p];
      else v *= cv[p];  // intersection: both sources are present
      c0 = C.a0[p];
      c1 = C.a1[p];
      if (C.a2) c2 = C.a2[p];
    }
    if (O.a0) O.a0[off + q] = c0;
    O.a1[off + q] = c1;
    if (O.a2) O.a2[off + q] = c2;
    ov[off + q] = v;
  }
}

// ---- CSR operands ----------------------------------------------------------

constexpr int kExpIPT = 8;
constexpr int kExpChunk = kExpIPT * kBlock;

// rows[p] = row of entry p of a CSR matrix, for a chunk of 2048 entries per workgroup:
// rows that start inside the chunk mark their first entry in LDS, every entry then takes
// the last mark at or before it (running maximum, rows ascend), entries before the first
// mark belong to the row cut by the chunk's start. Balanced for any row-length skew.
__global__ __launch_bounds__(kBlock) void expand_rows_kernel(int nnz, int nrows,
                                                             const int32_t* __restrict__ pos,
                                                             int32_t* __restrict__ rows) {
  __shared__ int32_t s_mark[kExpChunk];
  __shared__ int s_bounds[2];
  __shared__ int s_wmax[kBlock / kWave];
  const int base = blockIdx.x * kExpChunk;
  const int end = min(base + kExpChunk, nnz);
  // first row with pos > base, minus one = row holding entry `base`; likewise for the last entry
  if (wave_id() == 0) {
    const int r = wave_lower_bound(pos, nrows + 1, base + 1) - 1;
    if (lane_id() == 0) s_bounds[0] = r;
  } else if (wave_id() == 1) {
    const int r = wave_lower_bound(pos, nrows + 1, end) - 1;
    if (lane_id() == 0) s_bounds[1] = r;
  }
  for (int e = threadIdx.x; e < kExpChunk; e += kBlock) s_mark[e] = -1;
  __syncthreads();
  const int r_lo = s_bounds[0], r_hi = s_bounds[1];
  for (int r = r_lo + 1 + threadIdx.x; r <= r_hi; r += kBlock) {
    const int a = pos[r];
    if (pos[r + 1] > a) s_mark[a - base] = r;  // empty rows own no entry
  }
  __syncthreads();
  int32_t local[kExpIPT];
  int run = -1;
#pragma unroll
  for (int k = 0; k < kExpIPT; ++k) {
    const int m = s_mark[threadIdx.x * kExpIPT + k];
    run = m > run ? m : run;
    local[k] = run;
  }
  // exclusive running maximum over the threads before this one
  int inc = run;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int u = __shfl_up(inc, d);
    if (lane_id() >= d) inc = u > inc ? u : inc;
  }
  if (lane_id() == kWave - 1) s_wmax[wave_id()] = inc;
  __syncthreads();
  int before = __shfl_up(inc, 1);
  if (lane_id() == 0) before = -1;
  for (int w = 0; w < wave_id(); ++w) before = s_wmax[w] > before ? s_wmax[w] : before;
  if (before < r_lo) before = r_lo;
#pragma unroll
  for (int k = 0; k < kExpIPT; ++k) {
    const int p = base + threadIdx.x * kExpIPT + k;
    if (p < end) rows[p] = local[k] > before ? local[k] : before;
  }
}

__global__ __launch_bounds__(kBlock) void add_zero_i32_kernel(int32_t* __restrict__ out, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < n) out[i] = 0;
}

// ---- host ------------------------------------------------------------------

// parent[p] = index of the pos segment that holds position p (the row of a CSR entry, the
// column of a CSC entry); used by other translation units as well
spt_status launch_expand_parents(int n, int nparents, const int32_t* pos, int32_t* out, hipStream_t s) {
  if (n <= 0) return SPT_OK;
  hipLaunchKernelGGL(expand_rows_kernel, dim3((n + kExpChunk - 1) / kExpChunk), dim3(kBlock), 0, s, n,
                     nparents, pos, out);
  SPT_CHECK_LAUNCH("expand parents");
  return SPT_OK;
}

static int64_t add_tiles(int64_t nb, int64_t nc) { return (nb + nc + kAddTile - 1) / kAddTile; }

// fb / fc: formats of the operands (matrices may mix CSR and COO; the result takes B's format)
size_t add_workspace(Format fb, Format fc, const spt_tensor* B, const spt_tensor* C) {
  const int64_t nb = B->nvals, nc = C->nvals, nt = add_tiles(nb, nc);
  size_t n = 3 * align_up(static_cast<size_t>(nt + 1) * 4, 256) +
             align_up(static_cast<size_t>(nt) * kAddTile * 4, 256) + scan_workspace(nt) + 256;
  if (fb == Format::CSR)
    n += align_up(static_cast<size_t>(nb) * 4, 256) + align_up(static_cast<size_t>(nb + nc) * 4, 256);
  if (fc == Format::CSR) n += align_up(static_cast<size_t>(nc) * 4, 256);
  return n;
}

template <typename T, bool UNION>
static spt_status add_typed(Format fb, Format fc, const spt_tensor* B, const spt_tensor* C,
                            int32_t* out_pos, int32_t* out_crd0, int32_t* out_crd1, int32_t* out_crd2,
                            T* out_vals, int64_t* out_nnz, void* ws, size_t ws_bytes, hipStream_t s) {
  const int64_t nb64 = B->nvals, nc64 = C->nvals;
  if (nb64 + nc64 + kAddTile >= INT32_MAX)
    return fail(SPT_ERR_UNSUPPORTED, "add: more than 2^31 entries in both operands together");
  const int nb = static_cast<int>(nb64), nc = static_cast<int>(nc64);
  // an intersection with an empty operand is empty: no tile to walk
  const int ntiles = (!UNION && (nb == 0 || nc == 0)) ? 0 : static_cast<int>(add_tiles(nb, nc));
  const int64_t N = B->level[0].N;
  if (fb == Format::CSR) {
    if (N + 1 >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "add: too many rows");
    hipLaunchKernelGGL(add_zero_i32_kernel, dim3(static_cast<unsigned>((N + 1 + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, out_pos, N + 1);
    SPT_CHECK_LAUNCH("add zero pos");
  }
  if (ntiles == 0) {
    hipLaunchKernelGGL(add_total_kernel, dim3(1), dim3(kWave), 0, s, 0, nullptr, nullptr, out_nnz);
    SPT_CHECK_LAUNCH("add total");
    return SPT_OK;
  }
  const size_t need = add_workspace(fb, fc, B, C);
  if (!ws || ws_bytes < need)
    return fail(SPT_ERR_WORKSPACE, "add: workspace of %zu bytes needed, %zu given", need, ws_bytes);
  Workspace W(ws, ws_bytes);
  int* xs = W.take<int>(static_cast<size_t>(ntiles) + 1);
  int32_t* counts = W.take<int32_t>(static_cast<size_t>(ntiles) + 1);
  int32_t* offs = W.take<int32_t>(static_cast<size_t>(ntiles) + 1);
  uint32_t* rec = W.take<uint32_t>(static_cast<size_t>(ntiles) * kAddTile);
  int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace(ntiles)));

  // coordinate lists of the operands: CSR rows are expanded, COO levels are used as they are
  auto coords_of = [&](Format f, const spt_tensor* X, int n, CoordArrays* out) -> spt_status {
    if (f == Format::CSR) {
      int32_t* rows = W.take<int32_t>(n);
      if (n > 0) {
        hipLaunchKernelGGL(expand_rows_kernel, dim3((n + kExpChunk - 1) / kExpChunk), dim3(kBlock), 0, s,
                           n, static_cast<int>(N), X->level[1].pos, rows);
        SPT_CHECK_LAUNCH("add expand rows");
      }
      *out = CoordArrays{rows, X->level[1].crd, nullptr};
    } else {
      *out = CoordArrays{X->level[0].crd, X->level[1].crd, f == Format::COO3 ? X->level[2].crd : nullptr};
    }
    return SPT_OK;
  };
  CoordArrays cb, cc;
  spt_status st = coords_of(fb, B, nb, &cb);
  if (st != SPT_OK) return st;
  st = coords_of(fc, C, nc, &cc);
  if (st != SPT_OK) return st;
  CoordOut co;
  if (fb == Format::CSR) co = CoordOut{W.take<int32_t>(static_cast<size_t>(nb) + nc), out_crd1, nullptr};
  else co = CoordOut{out_crd0, out_crd1, fb == Format::COO3 ? out_crd2 : nullptr};

  const int pgrid = (ntiles + 1 + kBlock - 1) / kBlock;
  const bool third = cb.a2 != nullptr;
  const int w1 = key_bits_of(B->level[1].N), w2 = third ? key_bits_of(B->level[2].N) : 0;
  if (key_bits_of(N) + w1 + w2 <= 63) {
    PackedLoader kb{cb.a0, cb.a1, cb.a2, w1 + w2, w2};
    PackedLoader kc{cc.a0, cc.a1, cc.a2, w1 + w2, w2};
    hipLaunchKernelGGL(merge_partition_kernel<PackedLoader>, dim3(pgrid), dim3(kBlock), 0, s, kb, kc,
                       nb, nc, ntiles, kAddTile, xs);
    hipLaunchKernelGGL((add_merge_kernel<PackedLoader, UNION>), dim3(ntiles), dim3(kBlock), 0, s, kb,
                       kc, nb, nc, xs, rec, counts);
  } else {
    TripleLoader kb{cb.a0, cb.a1, cb.a2};
    TripleLoader kc{cc.a0, cc.a1, cc.a2};
    hipLaunchKernelGGL(merge_partition_kernel<TripleLoader>, dim3(pgrid), dim3(kBlock), 0, s, kb, kc,
                       nb, nc, ntiles, kAddTile, xs);
    hipLaunchKernelGGL((add_merge_kernel<TripleLoader, UNION>), dim3(ntiles), dim3(kBlock), 0, s, kb,
                       kc, nb, nc, xs, rec, counts);
  }
  SPT_CHECK_LAUNCH("add merge");
  st = device_scan_i32<false>(counts, offs, ntiles, scan_tmp, s);
  if (st != SPT_OK) return st;
  hipLaunchKernelGGL(add_total_kernel, dim3(1), dim3(kWave), 0, s, ntiles, counts, offs, out_nnz);
  SPT_CHECK_LAUNCH("add total");
  hipLaunchKernelGGL((add_fill_kernel<T, UNION>), dim3(ntiles), dim3(kBlock), 0, s, xs, rec, counts,
                     offs, cb, static_cast<const T*>(B->vals), cc, static_cast<const T*>(C->vals), co,
                     out_vals);
  SPT_CHECK_LAUNCH("add fill");
  if (fb == Format::CSR)  // pos of the result from its ordered rows (zero-filled above: an empty result keeps it)
    return launch_pos_from_sorted_rows(co.a0, nb + nc, static_cast<int>(N), out_pos, s, out_nnz);
  return SPT_OK;
}

// op: 0 = addition (union merge), 1 = element-wise multiplication (intersection merge)
spt_status add_dispatch(int op, Format fb, Format fc, const spt_tensor* B, const spt_tensor* C,
                        int32_t* out_pos, int32_t* out_crd0, int32_t* out_crd1, int32_t* out_crd2,
                        void* out_vals, int64_t* out_nnz, void* ws, size_t ws_bytes, hipStream_t s) {
  if (B->dtype == SPT_F64) {
    double* ov = static_cast<double*>(out_vals);
    return op == 0 ? add_typed<double, true>(fb, fc, B, C, out_pos, out_crd0, out_crd1, out_crd2, ov,
                                             out_nnz, ws, ws_bytes, s)
                   : add_typed<double, false>(fb, fc, B, C, out_pos, out_crd0, out_crd1, out_crd2, ov,
                                              out_nnz, ws, ws_bytes, s);
  }
  float* ov = static_cast<float*>(out_vals);
  return op == 0 ? add_typed<float, true>(fb, fc, B, C, out_pos, out_crd0, out_crd1, out_crd2, ov,
                                          out_nnz, ws, ws_bytes, s)
                 : add_typed<float, false>(fb, fc, B, C, out_pos, out_crd0, out_crd1, out_crd2, ov,
                                           out_nnz, ws, ws_bytes, s);
}

}  // namespace spt
