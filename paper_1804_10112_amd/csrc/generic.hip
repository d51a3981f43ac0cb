// Kernels for ANY composition of the six level formats (Section 3.1, Table 2), gfx950.
//
// The named formats have their own kernels; every other legal composition (DCSR, CSC, a
// dense matrix, hashed rows or columns, ...) runs here, on a device-side reading of the
// level functions. The paper's generated code walks a hierarchy from the root (Figure 5);
// a GPU wants one lane per stored value, so the walk is inverted: lane p takes leaf
// position p, climbs to the root by each level's parent rule,
//     dense, range:       p_{k-1} = p_k / N_k            (coord_access is p_{k-1} * N_k + i_k)
//     singleton, offset:  p_{k-1} = p_k                  (pos_bounds is [p_{k-1}, p_{k-1} + 1))
//     compressed:         p_{k-1} = last q with pos[q] <= p_k   (pos_bounds is pos[q .. q+1))
//     hashed:             p_{k-1} = p_k / W_k            (pos_bounds is [p_{k-1} W_k, (p_{k-1}+1) W_k))
// and then reads the coordinates back down, where each level's coordinate may depend on the
// one or two levels above it (range bounds from offset[i_{k-1}], offset level
// i_{k-1} + offset[i_{k-2}]). Positions that hold no component (a negative singleton
// coordinate, an empty hash bucket, a dense cell outside a range level's bounds) are skipped.
#include "common.hpp"
#include "scan.hpp"

namespace spt {

struct GLevel {
  int32_t kind, mode;
  int64_t N, M;
  const int32_t *pos, *crd, *offset;
  int64_t stride;  // elements between consecutive positions in crd (1 unless interleaved)
};
struct GTensor {
  int32_t nlevels, order;
  GLevel L[4];
};

static GTensor make_gtensor(const spt_tensor* T) {
  GTensor G;
  G.nlevels = T->nlevels;
  G.order = T->order;
  for (int k = 0; k < 4; ++k) {
    const spt_level& S = T->level[k < T->nlevels ? k : 0];
    G.L[k] = GLevel{S.kind, S.mode, S.N, S.M, S.pos, S.crd, S.offset, S.crd_stride > 1 ? S.crd_stride : 1};
  }
  return G;
}

// Last q in [0, m) with pos[q] <= p (pos has m + 1 ascending entries and pos[0] <= p < pos[m]).
__device__ __forceinline__ int64_t parent_in_pos(const int32_t* __restrict__ pos, int64_t m,
                                                 int64_t p) {
  int64_t lo = 0, hi = m;  // answer in [lo, hi)
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if (pos[mid] <= p) lo = mid; else hi = mid;
  }
  return lo;
}

// Coordinates of the component at leaf position p, by tensor dimension. False: no component.
__device__ __forceinline__ bool leaf_coordinates(const GTensor& G, int64_t p, int64_t* coord) {
  // loops over the four possible levels are fully unrolled with a level-count guard, so that
  // pk / ck stay in registers
  int64_t pk[4], ck[4] = {0, 0, 0, 0};
  const int nl = G.nlevels;
#pragma unroll
  for (int k = 0; k < 4; ++k) pk[k] = p;  // pk[nl - 1] = p; the levels above are overwritten below
#pragma unroll
  for (int k = 3; k >= 1; --k) {
    if (k <= nl - 1) {
      const GLevel& L = G.L[k];
      int64_t q;
      switch (L.kind) {
        case SPT_DENSE:
        case SPT_RANGE: q = pk[k] / L.N; break;
        case SPT_COMPRESSED: q = parent_in_pos(L.pos, L.M, pk[k]); break;
        case SPT_HASHED: q = pk[k] / L.M; break;
        default: q = pk[k];  // singleton, offset
      }
      pk[k - 1] = q;
    }
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if (k < nl) {
      const GLevel& L = G.L[k];
      int64_t c;
      switch (L.kind) {
        case SPT_DENSE: c = k == 0 ? pk[0] : pk[k] % L.N; break;
        case SPT_RANGE: {
          c = pk[k] % L.N;
          const int64_t off = L.offset[ck[k >= 1 ? k - 1 : 0]];
          const int64_t lo = off < 0 ? -off : 0, hi = L.M - off < L.N ? L.M - off : L.N;
          if (c < lo || c >= hi) return false;
          break;
        }
        case SPT_OFFSET: c = ck[k >= 1 ? k - 1 : 0] + L.offset[ck[k >= 2 ? k - 2 : 0]]; break;
        default:  // compressed, singleton, hashed: the stored coordinate
          c = L.crd[pk[k] * L.stride];
          if (c < 0) return false;
      }
      ck[k] = c;
      if (L.mode >= 0) coord[L.mode] = c;
    }
  }
  return true;
}

// ---- SpMV: one lane per stored value, one floating-point atomic per component ----

// A matrix has b1 = b2 = 1. A blocked matrix cast as a 4th-order tensor (Section 3.2) has
// dimensions (block rows, block columns, b1, b2), and component (i1, j1, i2, j2) is matrix
// element (i1 * b1 + i2, j1 * b2 + j2).
template <typename T>
__global__ __launch_bounds__(kBlock) void generic_spmv_kernel(const GTensor G, int64_t nvals,
                                                              int64_t b1, int64_t b2,
                                                              const T* __restrict__ vals,
                                                              const T* __restrict__ x,
                                                              T* __restrict__ y) {
  const int64_t p = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (p >= nvals) return;
  int64_t c[4] = {0, 0, 0, 0};
  if (leaf_coordinates(G, p, c))
    unsafeAtomicAdd(y + (c[0] * b1 + c[2]), vals[p] * x[c[1] * b2 + c[3]]);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void generic_zero_kernel(T* __restrict__ out, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < n) out[i] = T(0);
}

template <typename T>
static spt_status generic_spmv_typed(const spt_tensor* A, int64_t rows, int64_t b1, int64_t b2,
                                     const T* x, T* y, hipStream_t s) {
  if (rows > 0) {
    hipLaunchKernelGGL(generic_zero_kernel<T>, dim3(static_cast<unsigned>((rows + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, y, rows);
    SPT_CHECK_LAUNCH("generic zero");
  }
  if (A->nvals > 0) {
    hipLaunchKernelGGL(generic_spmv_kernel<T>,
                       dim3(static_cast<unsigned>((A->nvals + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                       s, make_gtensor(A), A->nvals, b1, b2, static_cast<const T*>(A->vals), x, y);
    SPT_CHECK_LAUNCH("generic spmv");
  }
  return SPT_OK;
}

// Size of tensor dimension `mode`: the N of the level that encodes it.
static int64_t mode_size(const spt_tensor* T, int mode) {
  for (int k = 0; k < T->nlevels; ++k)
    if (T->level[k].mode == mode) return T->level[k].N;
  return 0;
}

spt_status generic_spmv_dispatch(const spt_tensor* A, const void* x, void* y, hipStream_t s) {
  if (A->nvals >= (int64_t{1} << 40)) return fail(SPT_ERR_UNSUPPORTED, "spmv: tensor too large");
  const bool blocked = A->order == 4;
  const int64_t b1 = blocked ? mode_size(A, 2) : 1, b2 = blocked ? mode_size(A, 3) : 1;
  const int64_t rows = mode_size(A, 0) * b1;
  if (rows >= INT32_MAX || mode_size(A, 1) * b2 >= INT32_MAX)
    return fail(SPT_ERR_UNSUPPORTED, "spmv: matrix beyond 2^31 rows or columns");
  if (A->dtype == SPT_F64)
    return generic_spmv_typed<double>(A, rows, b1, b2, static_cast<const double*>(x),
                                      static_cast<double*>(y), s);
  return generic_spmv_typed<float>(A, rows, b1, b2, static_cast<const float*>(x),
                                   static_cast<float*>(y), s);
}

// ---- element-wise with a dense operand or a dense result ----

// out[p] = vals[p] * D(i, j) on the structure of the sparse operand (Figure 1); positions that
// hold no component give 0.
template <typename T>
__global__ __launch_bounds__(kBlock) void generic_mul_dense_kernel(const GTensor G, int64_t nvals,
                                                                   const T* __restrict__ vals,
                                                                   const T* __restrict__ D, int64_t ld,
                                                                   T* __restrict__ out) {
  const int64_t p = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (p >= nvals) return;
  int64_t c[4] = {0, 0, 0, 0};
  out[p] = leaf_coordinates(G, p, c) ? vals[p] * D[c[0] * ld + c[1]] : T(0);
}

// A(i, j) += v for every component: insertion into a dense result (Table 3: a dense level
// supports insert, its position is i * ld + j), so the operands need no merge.
template <typename T>
__global__ __launch_bounds__(kBlock) void generic_add_to_dense_kernel(const GTensor G, int64_t nvals,
                                                                      const T* __restrict__ vals,
                                                                      T* __restrict__ A, int64_t ld) {
  const int64_t p = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (p >= nvals) return;
  int64_t c[4] = {0, 0, 0, 0};
  if (leaf_coordinates(G, p, c)) unsafeAtomicAdd(A + (c[0] * ld + c[1]), vals[p]);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void generic_zero_rows_kernel(T* __restrict__ A, int64_t rows,
                                                                   int64_t cols, int64_t ld) {
  const int64_t q = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (q < rows * cols) A[(q / cols) * ld + q % cols] = T(0);
}

template <typename T>
static spt_status mul_dense_typed(const spt_tensor* B, const T* D, int64_t ld, T* out, hipStream_t s) {
  if (B->nvals == 0) return SPT_OK;
  hipLaunchKernelGGL(generic_mul_dense_kernel<T>,
                     dim3(static_cast<unsigned>((B->nvals + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                     make_gtensor(B), B->nvals, static_cast<const T*>(B->vals), D, ld, out);
  SPT_CHECK_LAUNCH("mul_dense");
  return SPT_OK;
}

spt_status mul_dense_dispatch(const spt_tensor* B, const void* D, int64_t ld, void* out, hipStream_t s) {
  if (B->nvals >= (int64_t{1} << 40)) return fail(SPT_ERR_UNSUPPORTED, "mul_dense: tensor too large");
  if (B->dtype == SPT_F64)
    return mul_dense_typed<double>(B, static_cast<const double*>(D), ld, static_cast<double*>(out), s);
  return mul_dense_typed<float>(B, static_cast<const float*>(D), ld, static_cast<float*>(out), s);
}

template <typename T>
static spt_status add_to_dense_typed(const spt_tensor* B, const spt_tensor* C, T* A, int64_t ld,
                                     hipStream_t s) {
  const int64_t rows = mode_size(B, 0), cols = mode_size(B, 1);
  if (rows * cols > 0) {
    hipLaunchKernelGGL(generic_zero_rows_kernel<T>,
                       dim3(static_cast<unsigned>((rows * cols + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                       s, A, rows, cols, ld);
    SPT_CHECK_LAUNCH("add_to_dense zero");
  }
  for (const spt_tensor* X : {B, C}) {
    if (X->nvals == 0) continue;
    hipLaunchKernelGGL(generic_add_to_dense_kernel<T>,
                       dim3(static_cast<unsigned>((X->nvals + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                       make_gtensor(X), X->nvals, static_cast<const T*>(X->vals), A, ld);
    SPT_CHECK_LAUNCH("add_to_dense");
  }
  return SPT_OK;
}

spt_status add_to_dense_dispatch(const spt_tensor* B, const spt_tensor* C, void* A, int64_t ld,
                                 hipStream_t s) {
  const int64_t rows = mode_size(B, 0), cols = mode_size(B, 1);
  if (B->nvals >= (int64_t{1} << 40) || C->nvals >= (int64_t{1} << 40) ||
      rows * cols >= (int64_t{1} << 40))
    return fail(SPT_ERR_UNSUPPORTED, "add_to_dense: operands or result too large");
  if (B->dtype == SPT_F64) return add_to_dense_typed<double>(B, C, static_cast<double*>(A), ld, s);
  return add_to_dense_typed<float>(B, C, static_cast<float*>(A), ld, s);
}

// ---- any format -> COO, in storage order (count per chunk, scan, fill) ----

constexpr int kCooChunk = kBlock;  // one leaf per lane

__global__ __launch_bounds__(kBlock) void to_coo_count_kernel(const GTensor G, int64_t nvals,
                                                              int32_t* __restrict__ counts) {
  const int64_t p = static_cast<int64_t>(blockIdx.x) * kCooChunk + threadIdx.x;
  int64_t c[4];
  const int has = (p < nvals && leaf_coordinates(G, p, c)) ? 1 : 0;
  int total;
  block_inclusive_sum(has, &total);
  if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

template <typename VT>
__global__ __launch_bounds__(kBlock) void to_coo_fill_kernel(const GTensor G, int64_t nvals,
                                                             int64_t b1, int64_t b2,
                                                             const VT* __restrict__ vals,
                                                             const int32_t* __restrict__ offs,
                                                             int32_t* __restrict__ o0,
                                                             int32_t* __restrict__ o1,
                                                             int32_t* __restrict__ o2,
                                                             VT* __restrict__ ov) {
  const int64_t p = static_cast<int64_t>(blockIdx.x) * kCooChunk + threadIdx.x;
  int64_t c[4] = {0, 0, 0, 0};
  const int has = (p < nvals && leaf_coordinates(G, p, c)) ? 1 : 0;
  int total;
  const int slot = offs[blockIdx.x] + block_inclusive_sum(has, &total) - has;
  if (has) {
    if (G.order == 4) {  // blocked matrix: element (i1 * b1 + i2, j1 * b2 + j2)
      o0[slot] = static_cast<int32_t>(c[0] * b1 + c[2]);
      o1[slot] = static_cast<int32_t>(c[1] * b2 + c[3]);
    } else {
      o0[slot] = static_cast<int32_t>(c[0]);
      if (G.order > 1) o1[slot] = static_cast<int32_t>(c[1]);
      if (G.order > 2) o2[slot] = static_cast<int32_t>(c[2]);
    }
    ov[slot] = vals[p];
  }
}

__global__ void to_coo_total_kernel(int nch, const int32_t* __restrict__ counts,
                                    const int32_t* __restrict__ offs, int64_t* __restrict__ out) {
  if (threadIdx.x == 0 && blockIdx.x == 0)
    *out = nch > 0 ? static_cast<int64_t>(offs[nch - 1]) + counts[nch - 1] : 0;
}

size_t to_coo_workspace(int64_t nvals) {
  const int64_t nch = (nvals + kCooChunk - 1) / kCooChunk;
  return 2 * align_up(static_cast<size_t>(nch + 1) * 4, 256) + scan_workspace(nch) + 256;
}

template <typename VT>
static spt_status to_coo_typed(const spt_tensor* T, int32_t* o0, int32_t* o1, int32_t* o2, VT* ov,
                               int64_t* out_nnz, void* ws, size_t ws_bytes, hipStream_t s) {
  const int64_t nvals = T->nvals;
  const int64_t nch64 = (nvals + kCooChunk - 1) / kCooChunk;
  if (nvals >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "to_coo: more than 2^31 leaf positions");
  const int nch = static_cast<int>(nch64);
  if (nch == 0) {
    hipLaunchKernelGGL(to_coo_total_kernel, dim3(1), dim3(kWave), 0, s, 0, nullptr, nullptr, out_nnz);
    SPT_CHECK_LAUNCH("to_coo total");
    return SPT_OK;
  }
  if (!ws || ws_bytes < to_coo_workspace(nvals))
    return fail(SPT_ERR_WORKSPACE, "to_coo: workspace of %zu bytes needed, %zu given",
                to_coo_workspace(nvals), ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* counts = W.take<int32_t>(nch + 1);
  int32_t* offs = W.take<int32_t>(nch + 1);
  int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace(nch)));
  const GTensor G = make_gtensor(T);
  hipLaunchKernelGGL(to_coo_count_kernel, dim3(nch), dim3(kBlock), 0, s, G, nvals, counts);
  SPT_CHECK_LAUNCH("to_coo count");
  spt_status st = device_scan_i32<false>(counts, offs, nch, scan_tmp, s);
  if (st != SPT_OK) return st;
  hipLaunchKernelGGL(to_coo_total_kernel, dim3(1), dim3(kWave), 0, s, nch, counts, offs, out_nnz);
  SPT_CHECK_LAUNCH("to_coo total");
  const bool blocked = T->order == 4;
  const int64_t b1 = blocked ? mode_size(T, 2) : 1, b2 = blocked ? mode_size(T, 3) : 1;
  if (blocked && (mode_size(T, 0) * b1 >= INT32_MAX || mode_size(T, 1) * b2 >= INT32_MAX))
    return fail(SPT_ERR_UNSUPPORTED, "to_coo: blocked matrix beyond 2^31 rows or columns");
  hipLaunchKernelGGL(to_coo_fill_kernel<VT>, dim3(nch), dim3(kBlock), 0, s, G, nvals, b1, b2,
                     static_cast<const VT*>(T->vals), offs, o0, o1, o2, ov);
  SPT_CHECK_LAUNCH("to_coo fill");
  return SPT_OK;
}

spt_status to_coo_dispatch(const spt_tensor* T, int32_t* o0, int32_t* o1, int32_t* o2, void* ov,
                           int64_t* out_nnz, void* ws, size_t ws_bytes, hipStream_t s) {
  if (T->dtype == SPT_F64)
    return to_coo_typed<uint64_t>(T, o0, o1, o2, static_cast<uint64_t*>(ov), out_nnz, ws, ws_bytes, s);
  return to_coo_typed<uint32_t>(T, o0, o1, o2, static_cast<uint32_t*>(ov), out_nnz, ws, ws_bytes, s);
}

}  // namespace spt
