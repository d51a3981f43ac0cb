// SpMV on BCSR, gfx950.
//
// Section 3.2 casts a blocked matrix format as a higher-order tensor: BCSR is the 4th-order
// composition (dense block rows, compressed block columns, dense rows in the block, dense
// columns in the block), one dense b1 x b2 block of values per stored block coordinate, and
//     y(i1, i2) = sum_{j1, j2} A(i1, j1, i2, j2) x(j1, j2)
// with y and x stored flat (element i1*b1 + i2, j1*b2 + j2). The values are one contiguous
// stream of b1*b2 numbers per block and 4 bytes of index per block, so the kernel is bound
// by reading that stream once at full width:
//   * a workgroup owns a chunk of consecutive blocks (block-balanced, whatever the lengths of
//     the block rows); the block rows that start in each chunk are found beforehand by one
//     bisection of pos per chunk boundary;
//   * consecutive lanes take consecutive 16-byte pieces of the chunk's values (where b2
//     values fill 1, 2 or 4 such pieces; otherwise lane q takes the b2 values of (block,
//     row-in-block) pair q), multiply them with the entries of x under the block's column
//     (block columns staged in LDS) and add the pieces of one pair across lanes;
//   * the pair's dot product goes to LDS, transposed to [row-in-block][block];
//   * one lane per (block row, row-in-block) then adds up its blocks from LDS. Rows that lie
//     inside the chunk are stored; the row that continues from the chunk before and the row
//     that continues into the next one leave the workgroup as carries, which a second small
//     kernel adds up in chunk order. No atomics: the result does not depend on scheduling.
#include "common.hpp"

namespace spt {

constexpr int kBcPairs = 2048;  // (block, row-in-block) pairs per workgroup
constexpr int kBcMaxEdge = 64;  // largest block edge this kernel takes

// row_start[c] = first block row r with pos[r] >= c * CH (Nb if none, and for c = nchunks):
// chunk c owns the block rows [row_start[c], row_start[c + 1]), those that start inside it,
// and the last chunk also takes the empty rows after the last block.
__global__ __launch_bounds__(kBlock) void bcsr_chunk_rows_kernel(int Nb, int CH, int nchunks,
                                                                 const int32_t* __restrict__ pos,
                                                                 int32_t* __restrict__ row_start) {
  const int c = blockIdx.x * kBlock + threadIdx.x;
  if (c > nchunks) return;
  int lo = 0, hi = Nb;  // answer in [lo, hi]
  const int64_t target = static_cast<int64_t>(c) * CH;
  if (c == nchunks) lo = Nb;
  while (lo < hi) {
    const int mid = lo + ((hi - lo) >> 1);
    if (pos[mid] < target) lo = mid + 1; else hi = mid;
  }
  row_start[c] = lo;
}

// carry layout: plane ii holds 2 slots per chunk, index ii * 2 * nchunks + 2 * chunk + slot;
// slot 0 = the part of the row that continues from the chunk before (never the first part of
// a row), slot 1 = the first part of a row that continues into the next chunk; key = scalar
// row (block row * b1 + ii) or -1.
template <typename T, int CB>
__global__ __launch_bounds__(kBlock) void bcsr_spmv_kernel(
    int64_t nblocks, int Nb, int R, int cb_rt, int CH, int nchunks,
    const int32_t* __restrict__ pos, const int32_t* __restrict__ row_start,
    const int32_t* __restrict__ crd, const T* __restrict__ vals, const T* __restrict__ x,
    T* __restrict__ y, int32_t* __restrict__ carry_key, T* __restrict__ carry_val) {
  extern __shared__ __align__(16) unsigned char bc_smem[];
  T* sDot = reinterpret_cast<T*>(bc_smem);  // R planes of CH + 1 dot products
  int32_t* sCrd = reinterpret_cast<int32_t*>(sDot + static_cast<size_t>(R) * (CH + 1));  // CH columns
  const int cb = CB > 0 ? CB : cb_rt;
  const int c = xcd_contiguous_block_id();
  const int64_t b0 = static_cast<int64_t>(c) * CH;
  const int64_t left = nblocks - b0;
  const int nb = left < CH ? static_cast<int>(left > 0 ? left : 0) : CH;
  const int plane = CH + 1;

  const int r_lo = row_start[c], r_hi = row_start[c + 1];  // rows that start inside the chunk

  // the chunk's block columns go through LDS: every lane of a block needs the same one, and
  // the loads of x then do not wait behind a load of their own index
  for (int k = threadIdx.x; k < nb; k += kBlock) sCrd[k] = crd[b0 + k];
  __syncthreads();

  // dot product of every (block, row-in-block) pair with the entries of x under the block
  const int npairs = nb * R;
  constexpr int EPV = 16 / static_cast<int>(sizeof(T));  // values per 16-byte load
  constexpr int VPR = CB / EPV > 0 ? CB / EPV : 1;       // 16-byte loads per pair
  if (CB >= EPV && CB % EPV == 0 && (VPR == 1 || VPR == 2 || VPR == 4)) {
    // consecutive lanes take consecutive 16-byte pieces of the value stream; the VPR lanes
    // of one pair then add up their pieces
    const int nvec = npairs * VPR;
    const T* base = vals + b0 * R * cb;
    constexpr int U = 4;  // pieces in flight per lane
    // (block, row-in-block) of this lane's piece, advanced by additions only: a division per
    // piece would cost more issue slots than the loads it serves
    constexpr int kStepQ = kBlock / VPR;
    const int dbl = kStepQ / R, dii = kStepQ - dbl * R;
    const int q0 = threadIdx.x / VPR, h = threadIdx.x - q0 * VPR;
    int bl = q0 / R, ii = q0 - bl * R;
    const int xoff = h * EPV;
    for (int e0 = threadIdx.x; e0 < nvec; e0 += U * kBlock) {
      int blu[U], iiu[U];
      int j1[U];
      T v[U][EPV], xv[U][EPV];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        blu[u] = bl;
        iiu[u] = ii;
        j1[u] = e0 + u * kBlock < nvec ? sCrd[bl] : 0;
        bl += dbl;
        ii += dii;
        if (ii >= R) {
          ii -= R;
          ++bl;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int e = e0 + u * kBlock;
        const T* pv = base + e * EPV;
#pragma unroll
        for (int k = 0; k < EPV; ++k) v[u][k] = e < nvec ? pv[k] : T(0);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const T* px = x + (j1[u] * cb + xoff);
#pragma unroll
        for (int k = 0; k < EPV; ++k) xv[u][k] = px[k];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        T d = T(0);
#pragma unroll
        for (int k = 0; k < EPV; ++k) d += v[u][k] * xv[u][k];
        if (VPR >= 2) d += __shfl_xor(d, 1);
        if (VPR >= 4) d += __shfl_xor(d, 2);
        if (h == 0 && e0 + u * kBlock < nvec) sDot[iiu[u] * plane + blu[u]] = d;
      }
    }
  } else {
    for (int q = threadIdx.x; q < npairs; q += kBlock) {
      const int bl = q / R, ii = q - bl * R;
      const int64_t j1 = sCrd[bl];
      const T* pv = vals + (b0 * R + q) * cb;
      const T* px = x + j1 * cb;
      T d = T(0);
      if (CB > 0) {
        T v[CB > 0 ? CB : 1], xv[CB > 0 ? CB : 1];
#pragma unroll
        for (int jj = 0; jj < CB; ++jj) v[jj] = pv[jj];
#pragma unroll
        for (int jj = 0; jj < CB; ++jj) xv[jj] = px[jj];
#pragma unroll
        for (int jj = 0; jj < CB; ++jj) d += v[jj] * xv[jj];
      } else {
        for (int jj = 0; jj < cb; ++jj) d += pv[jj] * px[jj];
      }
      sDot[ii * plane + bl] = d;
    }
  }
  __syncthreads();
  const int64_t e1 = b0 + nb;
  const int cstride = 2 * nchunks;

  // blocks [0, head) of the chunk belong to the row before r_lo, which began in an earlier chunk
  const int head = r_lo < Nb ? static_cast<int>((pos[r_lo] < e1 ? pos[r_lo] : e1) - b0) : nb;
  // the last row that starts here continues into the next chunk
  const bool tail = r_hi > r_lo && pos[r_hi] > e1;
  if (threadIdx.x < R) {
    const int ii = threadIdx.x;
    T s = T(0);
    for (int k = 0; k < head; ++k) s += sDot[ii * plane + k];
    const int slot = ii * cstride + 2 * c;
    carry_key[slot] = head > 0 ? (r_lo - 1) * R + ii : -1;
    carry_val[slot] = s;
    if (!tail) carry_key[slot + 1] = -1;
  }
  const int64_t nout = static_cast<int64_t>(r_hi - r_lo) * R;
  for (int64_t u = threadIdx.x; u < nout; u += kBlock) {
    const int rl = static_cast<int>(u / R), ii = static_cast<int>(u - static_cast<int64_t>(rl) * R);
    const int r = r_lo + rl;
    const int64_t p0 = pos[r], p1 = pos[r + 1];
    const int lo = static_cast<int>(p0 - b0);
    const int hi = static_cast<int>((p1 < e1 ? p1 : e1) - b0);
    T s = T(0);
    for (int k = lo; k < hi; ++k) s += sDot[ii * plane + k];
    if (p1 <= e1) {
      y[static_cast<int64_t>(r_lo) * R + u] = s;
    } else {  // only the last row of the chunk: its sum is completed from the carries
      const int slot = ii * cstride + 2 * c + 1;
      carry_key[slot] = r * R + ii;
      carry_val[slot] = s;
    }
  }
}

// One lane per (plane, chunk): a row's first part (slot 1) plus the parts of the chunks after
// it that continue the same row (their slot 0), added in chunk order.
template <typename T>
__global__ __launch_bounds__(kBlock) void bcsr_carry_kernel(int R, int nchunks,
                                                            const int32_t* __restrict__ carry_key,
                                                            const T* __restrict__ carry_val,
                                                            T* __restrict__ y) {
  const int64_t w = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (w >= static_cast<int64_t>(R) * nchunks) return;
  const int ii = static_cast<int>(w / nchunks), c = static_cast<int>(w - static_cast<int64_t>(ii) * nchunks);
  const int32_t* key = carry_key + static_cast<int64_t>(ii) * 2 * nchunks;
  const T* val = carry_val + static_cast<int64_t>(ii) * 2 * nchunks;
  const int32_t k = key[2 * c + 1];
  if (k < 0) return;
  T s = val[2 * c + 1];
  for (int d = c + 1; d < nchunks && key[2 * d] == k; ++d) s += val[2 * d];
  y[k] = s;
}

static int bcsr_chunk_blocks(int R) { return kBcPairs / R > 0 ? kBcPairs / R : 1; }

static int64_t bcsr_blocks(const spt_tensor* A) {
  const int64_t cells = A->level[2].N * A->level[3].N;
  return cells > 0 ? A->nvals / cells : 0;
}

static int64_t bcsr_chunks(const spt_tensor* A) {
  const int CH = bcsr_chunk_blocks(static_cast<int>(A->level[2].N));
  const int64_t n = (bcsr_blocks(A) + CH - 1) / CH;
  return n > 0 ? n : 1;
}

bool bcsr_fast_ok(const spt_tensor* A) {
  return A->level[2].N >= 1 && A->level[2].N <= kBcMaxEdge && A->level[3].N >= 1 &&
         A->level[3].N <= kBcMaxEdge;
}

size_t bcsr_workspace(const spt_tensor* A) {
  const size_t slots = static_cast<size_t>(2 * bcsr_chunks(A) * A->level[2].N);
  return align_up(slots * 4, 256) + align_up(slots * 8, 256) +
         align_up(static_cast<size_t>(bcsr_chunks(A) + 1) * 4, 256);
}

template <typename T, int CB>
static void bcsr_launch(int64_t nblocks, int Nb, int R, int cb, int CH, int nchunks,
                        const spt_tensor* A, const int32_t* row_start, const T* x, T* y, int32_t* ck,
                        T* cv, hipStream_t s) {
  const size_t lds = static_cast<size_t>(R) * (CH + 1) * sizeof(T) + static_cast<size_t>(CH) * 4;
  hipLaunchKernelGGL((bcsr_spmv_kernel<T, CB>), dim3(nchunks), dim3(kBlock), lds, s, nblocks, Nb,
                     R, cb, CH, nchunks, A->level[1].pos, row_start, A->level[1].crd,
                     static_cast<const T*>(A->vals), x, y, ck, cv);
}

template <typename T>
static spt_status bcsr_typed(const spt_tensor* A, const T* x, T* y, void* ws, size_t ws_bytes,
                             hipStream_t s) {
  const int64_t Nb64 = A->level[0].N, b1 = A->level[2].N, b2 = A->level[3].N;
  const int64_t nblocks = bcsr_blocks(A);
  if (A->nvals != nblocks * b1 * b2)
    return fail(SPT_ERR_INVALID_ARG, "BCSR: nvals must be a multiple of the block size b1*b2");
  if (Nb64 * b1 >= INT32_MAX || A->level[1].N * b2 >= INT32_MAX || nblocks >= INT32_MAX)
    return fail(SPT_ERR_UNSUPPORTED, "BCSR: matrix beyond 2^31 rows, columns or blocks");
  if (Nb64 == 0) return SPT_OK;
  const int Nb = static_cast<int>(Nb64), R = static_cast<int>(b1), cb = static_cast<int>(b2);
  const int CH = bcsr_chunk_blocks(R);
  const int64_t nch64 = bcsr_chunks(A);
  if (nch64 * 2 * R >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "BCSR: too many blocks");
  const int nchunks = static_cast<int>(nch64);
  const size_t need = bcsr_workspace(A);
  if (!ws || ws_bytes < need)
    return fail(SPT_ERR_WORKSPACE, "spmv (BCSR): workspace of %zu bytes needed, %zu given", need,
                ws_bytes);
  Workspace W(ws, ws_bytes);
  const size_t slots = static_cast<size_t>(2) * nchunks * R;
  int32_t* ck = W.take<int32_t>(slots);
  T* cv = reinterpret_cast<T*>(W.take<double>(slots));
  int32_t* rs = W.take<int32_t>(static_cast<size_t>(nchunks) + 1);
  hipLaunchKernelGGL(bcsr_chunk_rows_kernel, dim3((nchunks + 1 + kBlock - 1) / kBlock), dim3(kBlock), 0,
                     s, Nb, CH, nchunks, A->level[1].pos, rs);
  SPT_CHECK_LAUNCH("bcsr chunk rows");
  // b2 known at compile time for the common block widths: the run of b2 values and of x is
  // then read with the widest loads (the hardware takes them at any 4-byte alignment)
#define SPT_BCSR_CASE(CBV)                                                          \
  case CBV:                                                                         \
    bcsr_launch<T, CBV>(nblocks, Nb, R, cb, CH, nchunks, A, rs, x, y, ck, cv, s);      \
    break;
  switch (cb) {
    SPT_BCSR_CASE(1)
    SPT_BCSR_CASE(2)
    SPT_BCSR_CASE(3)
    SPT_BCSR_CASE(4)
    SPT_BCSR_CASE(6)
    SPT_BCSR_CASE(8)
    default:
      bcsr_launch<T, 0>(nblocks, Nb, R, cb, CH, nchunks, A, rs, x, y, ck, cv, s);
  }
#undef SPT_BCSR_CASE
  SPT_CHECK_LAUNCH("bcsr spmv");
  const int64_t nc = static_cast<int64_t>(R) * nchunks;
  hipLaunchKernelGGL(bcsr_carry_kernel<T>, dim3(static_cast<unsigned>((nc + kBlock - 1) / kBlock)),
                     dim3(kBlock), 0, s, R, nchunks, ck, cv, y);
  SPT_CHECK_LAUNCH("bcsr carries");
  return SPT_OK;
}

spt_status bcsr_spmv_dispatch(const spt_tensor* A, const void* x, void* y, void* ws, size_t ws_bytes,
                              hipStream_t s) {
  if (A->dtype == SPT_F64)
    return bcsr_typed<double>(A, static_cast<const double*>(x), static_cast<double*>(y), ws,
                              ws_bytes, s);
  return bcsr_typed<float>(A, static_cast<const float*>(x), static_cast<float*>(y), ws, ws_bytes, s);
}

}  // namespace spt
