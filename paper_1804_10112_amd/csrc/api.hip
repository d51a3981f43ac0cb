// C ABI entry points of libspt: descriptor validation, recognition of the level
// composition (Section 3.1: formats are compositions of level formats) and
// dispatch to the kernels. Host code only.
#include <cstring>

#include "common.hpp"

namespace spt {

static thread_local char g_err[512] = "";

void clear_error() { g_err[0] = 0; }

spt_status fail(spt_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

// implemented in the kernel translation units
spt_status spmv_dispatch(Format f, const spt_tensor* A, const void* x, void* y, void* ws,
                         size_t ws_bytes, hipStream_t s);
size_t seg_spmv_workspace(int64_t nnz);
size_t dcsr_spmv_workspace(const spt_tensor* A);
size_t csc_spmv_workspace(const spt_tensor* A);
spt_status aos_coo_spmv_dispatch(const spt_tensor* A, const void* x, void* y, void* ws,
                                 size_t ws_bytes, hipStream_t s);
size_t aos_coo_spmv_workspace(const spt_tensor* A);
spt_status spmv_sparse_x_dispatch(const spt_tensor* A, const spt_tensor* X, void* y, void* ws,
                                  size_t ws_bytes, hipStream_t s);
size_t coo_unordered_workspace(int dtype, int64_t nnz, int64_t nrows);
spt_status coo_to_csr_dispatch(const spt_tensor* A, int32_t order, int32_t* pos_out,
                               int32_t* crd_out, void* vals_out, void* ws, size_t ws_bytes,
                               hipStream_t s);
size_t coo_to_csr_workspace(const spt_tensor* A);
spt_status ttv_dispatch(Format f, const spt_tensor* B, const void* c, int32_t* out_crd0,
                        int32_t* out_crd1, void* out_vals, int64_t* out_nnz_dev, void* ws,
                        size_t ws_bytes, hipStream_t s);
size_t ttv_workspace(Format f, const spt_tensor* B);
spt_status mttkrp_dispatch(Format f, const spt_tensor* B, const void* C, const void* D, int32_t J,
                           void* A_out, void* ws, size_t ws_bytes, hipStream_t s);
size_t mttkrp_workspace(Format f, const spt_tensor* B, int32_t J);
spt_status spdm_dispatch(const spt_tensor* B, const void* C, int32_t J, void* A_out, void* ws,
                         size_t ws_bytes, hipStream_t s);

spt_status ttm_dispatch(Format f, const spt_tensor* B, const void* C, int32_t K, int32_t* out_crd0,
                        int32_t* out_crd1, void* out_vals, int64_t* out_nfib_dev, void* ws,
                        size_t ws_bytes, hipStream_t s);
size_t ttm_workspace(Format f, const spt_tensor* B, int32_t K);
spt_status innerprod_dispatch(Format f, const spt_tensor* B, const spt_tensor* C, void* out,
                              void* ws, size_t ws_bytes, hipStream_t s);
size_t innerprod_workspace(int64_t nb);

spt_status add_dispatch(int op, Format fb, Format fc, const spt_tensor* B, const spt_tensor* C,
                        int32_t* out_pos, int32_t* out_crd0, int32_t* out_crd1, int32_t* out_crd2,
                        void* out_vals, int64_t* out_nnz, void* ws, size_t ws_bytes, hipStream_t s);
size_t add_workspace(Format fb, Format fc, const spt_tensor* B, const spt_tensor* C);

spt_status pack_csf_dispatch(const spt_tensor* B, int32_t* pos0, int32_t* crd0, int32_t* pos1,
                             int32_t* crd1, int32_t* pos2, int32_t* crd2, void* vals_out,
                             int64_t* counts, void* ws, size_t ws_bytes, hipStream_t s);
size_t pack_csf_workspace(int64_t nnz);
spt_status pack_ell_dispatch(Format f, const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                             int32_t* longest, void* ws, size_t ws_bytes, hipStream_t s);
size_t pack_ell_workspace(Format f, const spt_tensor* A);
spt_status pack_hashed_dispatch(const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                                int32_t* dropped, hipStream_t s);
spt_status dia_offsets_dispatch(const spt_tensor* A, int32_t* offsets_out, int64_t cap, int64_t* K_dev,
                                void* ws, size_t ws_bytes, hipStream_t s);
size_t dia_offsets_workspace(const spt_tensor* A);
spt_status pack_dia_dispatch(const spt_tensor* A, int32_t K, const int32_t* offsets, void* vals_out,
                             hipStream_t s);

spt_status generic_spmv_dispatch(const spt_tensor* A, const void* x, void* y, hipStream_t s);
spt_status bcsr_spmv_dispatch(const spt_tensor* A, const void* x, void* y, void* ws, size_t ws_bytes,
                              hipStream_t s);
size_t bcsr_workspace(const spt_tensor* A);
bool bcsr_fast_ok(const spt_tensor* A);
spt_status to_coo_dispatch(const spt_tensor* T, int32_t* o0, int32_t* o1, int32_t* o2, void* ov,
                           int64_t* out_nnz, void* ws, size_t ws_bytes, hipStream_t s);
size_t to_coo_workspace(int64_t nvals);
spt_status mul_dense_dispatch(const spt_tensor* B, const void* D, int64_t ld, void* out, hipStream_t s);
spt_status add_to_dense_dispatch(const spt_tensor* B, const spt_tensor* C, void* A, int64_t ld,
                                 hipStream_t s);

spt_status validate_dispatch(const spt_tensor* T, int32_t* err, hipStream_t s);

static bool is(const spt_level& L, int kind) { return L.kind == kind; }
static bool unique(const spt_level& L) { return (L.flags & SPT_UNIQUE) != 0; }

// Table 1 legality and pointer/size checks for one level.
static bool level_ok(const spt_tensor* T, int k) {
  const spt_level& L = T->level[k];
  if (L.kind < SPT_DENSE || L.kind > SPT_HASHED) {
    fail(SPT_ERR_INVALID_ARG, "level %d: unknown level kind %d", k, L.kind);
    return false;
  }
  if (L.flags & ~(SPT_ORDERED | SPT_UNIQUE)) {
    fail(SPT_ERR_INVALID_ARG, "level %d: unknown property flags 0x%x", k, L.flags);
    return false;
  }
  if (L.kind == SPT_HASHED && (L.flags & SPT_ORDERED)) {
    fail(SPT_ERR_INVALID_ARG, "level %d: a hashed level cannot be ordered (Table 1)", k);
    return false;
  }
  if (L.N < 0 || L.M < 0 || L.crd_stride < 0) {
    fail(SPT_ERR_INVALID_ARG, "level %d: negative size or stride", k);
    return false;
  }
  if (L.mode < -1 || L.mode >= T->order) {
    fail(SPT_ERR_INVALID_ARG, "level %d: mode %d outside the tensor's %d dimensions", k, L.mode,
         T->order);
    return false;
  }
  const bool need_pos = L.kind == SPT_COMPRESSED;
  const bool need_crd = L.kind == SPT_COMPRESSED || L.kind == SPT_SINGLETON || L.kind == SPT_HASHED;
  const bool need_off = L.kind == SPT_RANGE || L.kind == SPT_OFFSET;
  if (need_pos && !L.pos) {
    fail(SPT_ERR_INVALID_ARG, "level %d: compressed level without pos", k);
    return false;
  }
  if (need_crd && !L.crd && T->nvals > 0) {
    fail(SPT_ERR_INVALID_ARG, "level %d: level without crd", k);
    return false;
  }
  if (need_off && !L.offset) {
    fail(SPT_ERR_INVALID_ARG, "level %d: range/offset level without offset", k);
    return false;
  }
  if ((L.kind == SPT_RANGE || L.kind == SPT_OFFSET) && k == 0) {
    fail(SPT_ERR_INVALID_ARG, "level %d: range/offset level needs an enclosing level", k);
    return false;
  }
  if (L.kind == SPT_SINGLETON && k == 0) {
    fail(SPT_ERR_INVALID_ARG, "level 0 cannot be a singleton level");
    return false;
  }
  return true;
}

Format recognize(const spt_tensor* T) {
  if (!T) {
    fail(SPT_ERR_INVALID_ARG, "null tensor descriptor");
    return Format::Invalid;
  }
  if (T->order < 1 || T->order > 4 || T->nlevels < 1 || T->nlevels > 4) {
    fail(SPT_ERR_INVALID_ARG, "order %d / nlevels %d out of range", T->order, T->nlevels);
    return Format::Invalid;
  }
  if (T->dtype != SPT_F32 && T->dtype != SPT_F64) {
    fail(SPT_ERR_INVALID_ARG, "unknown dtype %d", T->dtype);
    return Format::Invalid;
  }
  if (T->nvals < 0 || (T->nvals > 0 && !T->vals)) {
    fail(SPT_ERR_INVALID_ARG, "vals is null or nvals negative");
    return Format::Invalid;
  }
  for (int k = 0; k < T->nlevels; ++k)
    if (!level_ok(T, k)) return Format::Invalid;
  const spt_level* L = T->level;
  for (int k = 0; k < T->nlevels; ++k)
    if (L[k].crd_stride > 1) {  // interleaved coordinates: none of the format kernels reads them
      fail(SPT_ERR_UNSUPPORTED,
           "level %d has interleaved coordinates (crd_stride %lld): supported by spt_spmv, spt_to_coo, "
           "spt_mul_dense and spt_add_to_dense; spt_to_coo converts to contiguous coordinates",
           k, (long long)L[k].crd_stride);
      return Format::Unsupported;
    }
  auto modes = [&](int a, int b, int c, int d) {
    const int want[4] = {a, b, c, d};
    for (int k = 0; k < T->nlevels; ++k)
      if (L[k].mode != want[k]) return false;
    return true;
  };
  if (T->order == 2 && T->nlevels == 2) {
    if (is(L[0], SPT_DENSE) && is(L[1], SPT_COMPRESSED) && modes(0, 1, 0, 0)) {
      if (L[1].M != L[0].N) {
        fail(SPT_ERR_INVALID_ARG, "CSR: column level must have one parent per row (M = N rows)");
        return Format::Invalid;
      }
      return Format::CSR;
    }
    // CSC: the levels store the dimensions in the order (column, row); SpMV only
    if (is(L[0], SPT_DENSE) && is(L[1], SPT_COMPRESSED) && modes(1, 0, 0, 0) && L[1].M == L[0].N &&
        L[1].pos)
      return Format::CSC;
    // DCSR with unique rows has a fast path for SpMV; every other operation and DCSR with
    // repeated row coordinates take it as "any composition"
    if (is(L[0], SPT_COMPRESSED) && is(L[1], SPT_COMPRESSED) && modes(0, 1, 0, 0) && L[0].M == 1 &&
        unique(L[0]) && L[1].pos && (L[0].crd || L[1].M == 0)) {
      if (T->nvals > 0 && L[1].M < 1) {
        fail(SPT_ERR_INVALID_ARG, "DCSR: values are stored but the column level has no parent row (M = 0)");
        return Format::Invalid;
      }
      return Format::DCSR;
    }
    if (is(L[0], SPT_COMPRESSED) && is(L[1], SPT_SINGLETON) && modes(0, 1, 0, 0)) {
      if (L[0].M != 1) {
        fail(SPT_ERR_INVALID_ARG, "COO: the row level has one root parent (M = 1)");
        return Format::Invalid;
      }
      return Format::COO2;
    }
  }
  if (T->order == 2 && T->nlevels == 3) {
    if (is(L[0], SPT_DENSE) && is(L[1], SPT_RANGE) && is(L[2], SPT_OFFSET) && modes(-1, 0, 1, 0)) {
      if (L[1].offset != L[2].offset) {
        fail(SPT_ERR_INVALID_ARG, "DIA: range and offset level must share one offset array");
        return Format::Invalid;
      }
      if (T->nvals != L[0].N * L[1].N) {
        fail(SPT_ERR_INVALID_ARG, "DIA: nvals must be K*N");
        return Format::Invalid;
      }
      if (L[2].N != L[1].M) {
        fail(SPT_ERR_INVALID_ARG, "DIA: the range level's M must be the column dimension");
        return Format::Invalid;
      }
      return Format::DIA;
    }
    if (is(L[0], SPT_DENSE) && is(L[1], SPT_DENSE) && is(L[2], SPT_SINGLETON) &&
        modes(-1, 0, 1, 0)) {
      if (T->nvals != L[0].N * L[1].N) {
        fail(SPT_ERR_INVALID_ARG, "ELL: nvals must be W*N");
        return Format::Invalid;
      }
      return Format::ELL;
    }
  }
  if (T->order == 3 && T->nlevels == 3 && modes(0, 1, 2, 0)) {
    if (is(L[0], SPT_COMPRESSED) && is(L[1], SPT_SINGLETON) && is(L[2], SPT_SINGLETON)) {
      if (L[0].M != 1) {
        fail(SPT_ERR_INVALID_ARG, "COO: the first level has one root parent (M = 1)");
        return Format::Invalid;
      }
      return Format::COO3;
    }
    if (is(L[0], SPT_COMPRESSED) && is(L[1], SPT_COMPRESSED) && is(L[2], SPT_COMPRESSED)) {
      if (L[0].M != 1 || !unique(L[0]) || !unique(L[1])) {
        fail(SPT_ERR_INVALID_ARG, "CSF: root level needs M = 1 and the upper levels are unique");
        return Format::Invalid;
      }
      // M of a compressed level is the number of positions of its parent level (Section 3.1):
      // level 1 has one segment per stored slice, level 2 one per stored fibre. The kernels
      // bisect pos[0 .. M]; the host can only check that values imply parents
      // (spt_validate checks pos0[1] = M1, pos1[M1] = M2, pos2[M2] = nvals on the device).
      if (T->nvals > 0 && (L[1].M < 1 || L[2].M < 1)) {
        fail(SPT_ERR_INVALID_ARG, "CSF: values are stored but level 1 or 2 has no parent position (M = 0)");
        return Format::Invalid;
      }
      return Format::CSF3;
    }
  }
  if (T->order == 4 && T->nlevels == 4 && modes(0, 1, 2, 3) && is(L[0], SPT_DENSE) &&
      is(L[1], SPT_COMPRESSED) && is(L[2], SPT_DENSE) && is(L[3], SPT_DENSE)) {
    if (L[1].M != L[0].N) {
      fail(SPT_ERR_INVALID_ARG, "BCSR: block column level must have one parent per block row");
      return Format::Invalid;
    }
    return Format::BCSR;
  }
  fail(SPT_ERR_UNSUPPORTED,
       "level composition not supported (supported: CSR, COO, DIA, ELL, BCSR, 3rd-order COO, CSF)");
  return Format::Unsupported;
}

// Structural rules under which the per-value reading of the level functions is defined for
// a composition that has no kernel of its own. Call after recognize() returned a format or
// Unsupported (so every level passed level_ok). Sets the error and returns false otherwise.
static bool generic_ok(const spt_tensor* T) {
  const spt_level* L = T->level;
  if (!(L[0].kind == SPT_DENSE || L[0].kind == SPT_HASHED ||
        (L[0].kind == SPT_COMPRESSED && L[0].M == 1))) {
    fail(SPT_ERR_UNSUPPORTED, "level 0 must be dense, hashed or compressed with one parent (M = 1)");
    return false;
  }
  int seen[4] = {0, 0, 0, 0};
  for (int k = 0; k < T->nlevels; ++k) {
    if (L[k].kind == SPT_OFFSET && k < 2) {
      fail(SPT_ERR_UNSUPPORTED, "level %d: an offset level needs two levels above it", k);
      return false;
    }
    if (T->nvals > 0 && (((L[k].kind == SPT_DENSE || L[k].kind == SPT_RANGE) && L[k].N <= 0) ||
                         (L[k].kind == SPT_HASHED && L[k].M <= 0))) {
      fail(SPT_ERR_INVALID_ARG, "level %d: empty extent but values are stored", k);
      return false;
    }
    if (L[k].N >= INT32_MAX || L[k].M >= INT32_MAX) {
      fail(SPT_ERR_UNSUPPORTED, "level %d: extent beyond int32", k);
      return false;
    }
    if (L[k].mode >= 0) ++seen[L[k].mode];
  }
  for (int m = 0; m < T->order; ++m)
    if (seen[m] != 1) {
      fail(SPT_ERR_UNSUPPORTED, "tensor dimension %d must be encoded by exactly one level", m);
      return false;
    }
  clear_error();
  return true;
}

// The kernels carve typed arrays out of the workspace at 256-byte steps.
static bool ws_misaligned(const void* ws) {
  if (ws && reinterpret_cast<uintptr_t>(ws) % 256 != 0) {
    fail(SPT_ERR_INVALID_ARG, "workspace pointer is not 256-byte aligned");
    return true;
  }
  return false;
}

// An array-of-structs COO matrix: both levels read one array of (row, col) pairs.
static bool is_aos_coo_matrix(const spt_tensor* T) {
  const spt_level* L = T->level;
  return T->order == 2 && T->nlevels == 2 && L[0].kind == SPT_COMPRESSED && L[0].M == 1 &&
         L[1].kind == SPT_SINGLETON && L[0].mode == 0 && L[1].mode == 1 && L[0].crd_stride == 2 &&
         L[1].crd_stride == 2 && L[0].crd && L[1].crd == L[0].crd + 1 && T->nvals < INT32_MAX;
}

static spt_status status_of(Format f) {
  return f == Format::Invalid ? SPT_ERR_INVALID_ARG : SPT_ERR_UNSUPPORTED;
}

}  // namespace spt

using namespace spt;

extern "C" {

const char* spt_last_error(void) { return g_err; }
const char* spt_version(void) { return "spt 0.1 gfx950"; }

spt_status spt_spmv(const spt_tensor* A, const void* x, void* y, void* ws, size_t ws_bytes,
                    void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(A);
  if (f == Format::Invalid) return status_of(f);
  if (f == Format::Unsupported && is_aos_coo_matrix(A)) {
    clear_error();
    if (!x || !y) return fail(SPT_ERR_INVALID_ARG, "spmv: x or y is null");
    return aos_coo_spmv_dispatch(A, x, y, ws, ws_bytes, static_cast<hipStream_t>(stream));
  }
  if (f == Format::Unsupported || (f == Format::BCSR && !bcsr_fast_ok(A))) {
    // no kernel of its own: per-value reading of the level functions
    if (A->order != 2 && A->order != 4)
      return fail(SPT_ERR_UNSUPPORTED, "spmv: A must be a matrix or a blocked matrix of order 4");
    if (!generic_ok(A)) return SPT_ERR_UNSUPPORTED;
    if (!x || !y) return fail(SPT_ERR_INVALID_ARG, "spmv: x or y is null");
    return generic_spmv_dispatch(A, x, y, static_cast<hipStream_t>(stream));
  }
  if (!x || !y) return fail(SPT_ERR_INVALID_ARG, "spmv: x or y is null");
  if (f == Format::BCSR)
    return bcsr_spmv_dispatch(A, x, y, ws, ws_bytes, static_cast<hipStream_t>(stream));
  return spmv_dispatch(f, A, x, y, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

spt_status spt_validate(const spt_tensor* T, int32_t* err_dev, void* stream) {
  clear_error();
  Format f = recognize(T);
  if (f == Format::Invalid) return SPT_ERR_INVALID_ARG;
  if (f == Format::Unsupported && !generic_ok(T)) return SPT_ERR_UNSUPPORTED;
  clear_error();
  if (!err_dev) return fail(SPT_ERR_INVALID_ARG, "validate: err_dev is null");
  return validate_dispatch(T, err_dev, static_cast<hipStream_t>(stream));
}

spt_status spt_spmv_sparse_x(const spt_tensor* A, const spt_tensor* x, void* y, void* ws,
                             size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(A);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::CSR) return fail(SPT_ERR_UNSUPPORTED, "spmv_sparse_x: A must be CSR");
  if (!x || !y) return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: x or y is null");
  if (x->order != 1 || x->nlevels != 1)
    return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: x must be a 1st-order tensor of one level");
  if (x->dtype != A->dtype) return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: x and A differ in dtype");
  if (x->nvals < 0 || (x->nvals > 0 && !x->vals))
    return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: x.vals is null or nvals negative");
  const spt_level& L = x->level[0];
  if (L.mode != 0) return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: x's level must encode mode 0");
  if (L.kind == SPT_HASHED) {
    if (L.flags & SPT_ORDERED)
      return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: a hashed level cannot be ordered (Table 1)");
    if (!L.crd || L.M < 1 || x->nvals != L.M)
      return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: hashed x needs crd and nvals = W >= 1");
  } else if (L.kind == SPT_COMPRESSED) {
    if (!(L.flags & SPT_ORDERED) || !(L.flags & SPT_UNIQUE))
      return fail(SPT_ERR_UNSUPPORTED, "spmv_sparse_x: a sparse vector x must be ordered and unique");
    if (L.M != 1 || !L.pos || (!L.crd && x->nvals > 0))
      return fail(SPT_ERR_INVALID_ARG, "spmv_sparse_x: sparse vector x needs pos, crd and M = 1");
  } else {
    return fail(SPT_ERR_UNSUPPORTED, "spmv_sparse_x: x must be a compressed or a hashed level");
  }
  return spmv_sparse_x_dispatch(A, x, y, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

spt_status spt_coo_to_csr(const spt_tensor* A, int32_t order, int32_t* pos_out, int32_t* crd_out,
                          void* vals_out, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(A);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO2) return fail(SPT_ERR_UNSUPPORTED, "coo_to_csr: input is not a COO matrix");
  if (order != SPT_ORDER_ROW_COL && order != SPT_ORDER_ROW_STABLE)
    return fail(SPT_ERR_INVALID_ARG, "coo_to_csr: unknown order %d", order);
  if (!pos_out || ((!crd_out || !vals_out) && A->nvals > 0))
    return fail(SPT_ERR_INVALID_ARG, "coo_to_csr: null output");
  return coo_to_csr_dispatch(A, order, pos_out, crd_out, vals_out, ws, ws_bytes,
                             static_cast<hipStream_t>(stream));
}

spt_status spt_ttv(const spt_tensor* B, const void* c, int32_t* out_crd0, int32_t* out_crd1,
                   void* out_vals, int64_t* out_nnz_dev, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(B);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO3 && f != Format::CSF3)
    return fail(SPT_ERR_UNSUPPORTED, "ttv: input is not a 3rd-order COO or CSF tensor");
  if (!c || (!out_vals && B->nvals > 0)) return fail(SPT_ERR_INVALID_ARG, "ttv: null operand");
  if (f == Format::COO3 && (!out_nnz_dev || ((!out_crd0 || !out_crd1) && B->nvals > 0)))
    return fail(SPT_ERR_INVALID_ARG, "ttv: COO output needs out_crd0, out_crd1, out_nnz_dev");
  return ttv_dispatch(f, B, c, out_crd0, out_crd1, out_vals, out_nnz_dev, ws, ws_bytes,
                      static_cast<hipStream_t>(stream));
}

spt_status spt_mttkrp(const spt_tensor* B, const void* C, const void* D, int32_t J, void* A_out,
                      void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(B);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO3 && f != Format::CSF3)
    return fail(SPT_ERR_UNSUPPORTED, "mttkrp: input is not a 3rd-order COO or CSF tensor");
  if (J < 1 || J > 1024) return fail(SPT_ERR_INVALID_ARG, "mttkrp: J = %d outside [1,1024]", J);
  if (!C || !D || !A_out) return fail(SPT_ERR_INVALID_ARG, "mttkrp: null operand");
  return mttkrp_dispatch(f, B, C, D, J, A_out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

spt_status spt_spdm(const spt_tensor* B, const void* C, int32_t J, void* A_out, void* ws,
                    size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(B);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO2) return fail(SPT_ERR_UNSUPPORTED, "spdm: B must be a COO matrix");
  if (J < 1 || J > 1024) return fail(SPT_ERR_INVALID_ARG, "spdm: J = %d outside [1,1024]", J);
  if (!C || !A_out) return fail(SPT_ERR_INVALID_ARG, "spdm: null operand");
  return spdm_dispatch(B, C, J, A_out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

spt_status spt_ttm(const spt_tensor* B, const void* C, int32_t K, int32_t* out_crd0,
                   int32_t* out_crd1, void* out_vals, int64_t* out_nfib_dev, void* ws,
                   size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(B);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO3 && f != Format::CSF3)
    return fail(SPT_ERR_UNSUPPORTED, "ttm: B must be COO3 or CSF3");
  if (K < 1 || K > 1024) return fail(SPT_ERR_INVALID_ARG, "ttm: K = %d outside [1,1024]", K);
  if (!C || !out_vals) return fail(SPT_ERR_INVALID_ARG, "ttm: null operand");
  if (f == Format::COO3 && (!out_crd0 || !out_crd1 || !out_nfib_dev))
    return fail(SPT_ERR_INVALID_ARG, "ttm: COO output needs out_crd0, out_crd1 and out_nfib_dev");
  return ttm_dispatch(f, B, C, K, out_crd0, out_crd1, out_vals, out_nfib_dev, ws, ws_bytes,
                      static_cast<hipStream_t>(stream));
}

spt_status spt_innerprod(const spt_tensor* B, const spt_tensor* C, void* alpha_out, void* ws,
                         size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format fb = recognize(B);
  if (fb == Format::Invalid || fb == Format::Unsupported) return status_of(fb);
  Format fc = recognize(C);
  if (fc == Format::Invalid || fc == Format::Unsupported) return status_of(fc);
  if (fb != fc || (fb != Format::COO3 && fb != Format::COO2))
    return fail(SPT_ERR_UNSUPPORTED, "innerprod: B and C must both be COO3 or both COO matrices");
  if (B->dtype != C->dtype) return fail(SPT_ERR_INVALID_ARG, "innerprod: B and C differ in dtype");
  if (!alpha_out) return fail(SPT_ERR_INVALID_ARG, "innerprod: alpha_out is null");
  for (int k = 0; k < B->nlevels; ++k) {
    if (B->level[k].N != C->level[k].N)
      return fail(SPT_ERR_INVALID_ARG, "innerprod: dimension %d differs (%lld vs %lld)", k,
                  (long long)B->level[k].N, (long long)C->level[k].N);
    if (!(B->level[k].flags & C->level[k].flags & SPT_ORDERED))
      return fail(SPT_ERR_UNSUPPORTED, "innerprod: every level of B and C must be ordered");
  }
  return innerprod_dispatch(fb, B, C, alpha_out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

spt_status spt_coo3_to_csf(const spt_tensor* B, int32_t* pos0, int32_t* crd0, int32_t* pos1,
                           int32_t* crd1, int32_t* pos2, int32_t* crd2, void* vals_out,
                           int64_t* counts_dev, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(B);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO3) return fail(SPT_ERR_UNSUPPORTED, "coo3_to_csf: B must be COO3");
  for (int k = 0; k < 3; ++k)
    if (!(B->level[k].flags & SPT_ORDERED))
      return fail(SPT_ERR_UNSUPPORTED, "coo3_to_csf: every level of B must be ordered");
  if (!pos0 || !crd0 || !pos1 || !crd1 || !pos2 || !crd2 || !vals_out || !counts_dev)
    return fail(SPT_ERR_INVALID_ARG, "coo3_to_csf: null output");
  return pack_csf_dispatch(B, pos0, crd0, pos1, crd1, pos2, crd2, vals_out, counts_dev, ws, ws_bytes,
                           static_cast<hipStream_t>(stream));
}

spt_status spt_to_ell(const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                      int32_t* longest_dev, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(A);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO2 && f != Format::CSR)
    return fail(SPT_ERR_UNSUPPORTED, "to_ell: A must be a COO matrix or CSR");
  if (f == Format::COO2 && !(A->level[0].flags & A->level[1].flags & SPT_ORDERED))
    return fail(SPT_ERR_UNSUPPORTED, "to_ell: both levels of a COO source must be ordered");
  if (W < 0) return fail(SPT_ERR_INVALID_ARG, "to_ell: W = %d is negative", W);
  if (!longest_dev || (W > 0 && (!crd_out || !vals_out)))
    return fail(SPT_ERR_INVALID_ARG, "to_ell: null output");
  return pack_ell_dispatch(f, A, W, crd_out, vals_out, longest_dev, ws, ws_bytes,
                           static_cast<hipStream_t>(stream));
}

spt_status spt_to_hashed_rows(const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                              int32_t* dropped_dev, void* stream) {
  clear_error();
  Format f = recognize(A);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO2) return fail(SPT_ERR_UNSUPPORTED, "to_hashed_rows: A must be a COO matrix");
  if (W < 1) return fail(SPT_ERR_INVALID_ARG, "to_hashed_rows: W = %d, at least one slot per row needed", W);
  if (!crd_out || !vals_out || !dropped_dev) return fail(SPT_ERR_INVALID_ARG, "to_hashed_rows: null output");
  return pack_hashed_dispatch(A, W, crd_out, vals_out, dropped_dev, static_cast<hipStream_t>(stream));
}

spt_status spt_coo_dia_offsets(const spt_tensor* A, int32_t* offsets_out, int64_t cap,
                               int64_t* K_dev, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(A);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO2) return fail(SPT_ERR_UNSUPPORTED, "coo_dia_offsets: A must be a COO matrix");
  if (cap < 0 || !K_dev || (cap > 0 && !offsets_out))
    return fail(SPT_ERR_INVALID_ARG, "coo_dia_offsets: null output or negative capacity");
  return dia_offsets_dispatch(A, offsets_out, cap, K_dev, ws, ws_bytes,
                              static_cast<hipStream_t>(stream));
}

spt_status spt_coo_to_dia(const spt_tensor* A, int32_t K, const int32_t* offsets, void* vals_out,
                          void* stream) {
  clear_error();
  Format f = recognize(A);
  if (f == Format::Invalid || f == Format::Unsupported) return status_of(f);
  if (f != Format::COO2) return fail(SPT_ERR_UNSUPPORTED, "coo_to_dia: A must be a COO matrix");
  if (K < 0 || (K > 0 && (!offsets || !vals_out)))
    return fail(SPT_ERR_INVALID_ARG, "coo_to_dia: null array or negative K");
  return pack_dia_dispatch(A, K, offsets, vals_out, static_cast<hipStream_t>(stream));
}

spt_status spt_to_coo(const spt_tensor* T, int32_t* out_crd0, int32_t* out_crd1, int32_t* out_crd2,
                      void* out_vals, int64_t* out_nnz_dev, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format f = recognize(T);
  if (f == Format::Invalid) return status_of(f);
  if (!generic_ok(T)) return SPT_ERR_UNSUPPORTED;
  // a blocked matrix (order 4) is written as the matrix it stores: two coordinate arrays
  if (!out_nnz_dev || (T->nvals > 0 && (!out_crd0 || !out_vals || (T->order > 1 && !out_crd1) ||
                                        (T->order == 3 && !out_crd2))))
    return fail(SPT_ERR_INVALID_ARG, "to_coo: null output");
  return to_coo_dispatch(T, out_crd0, out_crd1, out_crd2, out_vals, out_nnz_dev, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

// Common operand checks of spt_add and spt_mul; returns both formats or sets the error.
// Matrices may mix CSR and COO (the result takes B's format); 3rd-order operands are both COO.
static spt_status add_operands(const spt_tensor* B, const spt_tensor* C, Format* fb_out,
                               Format* fc_out) {
  Format fb = recognize(B);
  if (fb == Format::Invalid || fb == Format::Unsupported) return status_of(fb);
  Format fc = recognize(C);
  if (fc == Format::Invalid || fc == Format::Unsupported) return status_of(fc);
  const bool mat_b = fb == Format::COO2 || fb == Format::CSR, mat_c = fc == Format::COO2 || fc == Format::CSR;
  if (!((mat_b && mat_c) || (fb == Format::COO3 && fc == Format::COO3)))
    return fail(SPT_ERR_UNSUPPORTED, "add/mul: B and C must be COO or CSR matrices, or both COO3");
  if (B->dtype != C->dtype) return fail(SPT_ERR_INVALID_ARG, "add/mul: B and C differ in dtype");
  for (int k = 0; k < B->nlevels; ++k) {
    if (B->level[k].N != C->level[k].N)
      return fail(SPT_ERR_INVALID_ARG, "add/mul: dimension %d differs (%lld vs %lld)", k,
                  (long long)B->level[k].N, (long long)C->level[k].N);
    // a dense row level is ordered by construction
    if (!(fb == Format::CSR && k == 0) && !(B->level[k].flags & SPT_ORDERED))
      return fail(SPT_ERR_UNSUPPORTED, "add/mul: every level of B must be ordered");
    if (!(fc == Format::CSR && k == 0) && !(C->level[k].flags & SPT_ORDERED))
      return fail(SPT_ERR_UNSUPPORTED, "add/mul: every level of C must be ordered");
  }
  *fb_out = fb;
  *fc_out = fc;
  return SPT_OK;
}

static spt_status add_or_mul(int op, const spt_tensor* B, const spt_tensor* C, int32_t* out_pos,
                             int32_t* out_crd0, int32_t* out_crd1, int32_t* out_crd2, void* out_vals,
                             int64_t* out_nnz_dev, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  if (ws_misaligned(ws)) return SPT_ERR_INVALID_ARG;
  Format fb, fc;
  spt_status st = add_operands(B, C, &fb, &fc);
  if (st != SPT_OK) return st;
  if (!out_crd1 || !out_vals || !out_nnz_dev)
    return fail(SPT_ERR_INVALID_ARG, "add/mul: out_crd1, out_vals and out_nnz_dev are required");
  if (fb == Format::CSR && !out_pos) return fail(SPT_ERR_INVALID_ARG, "add/mul: CSR result needs out_pos");
  if (fb != Format::CSR && !out_crd0) return fail(SPT_ERR_INVALID_ARG, "add/mul: COO result needs out_crd0");
  if (fb == Format::COO3 && !out_crd2) return fail(SPT_ERR_INVALID_ARG, "add/mul: COO3 result needs out_crd2");
  return add_dispatch(op, fb, fc, B, C, out_pos, out_crd0, out_crd1, out_crd2, out_vals, out_nnz_dev,
                      ws, ws_bytes, static_cast<hipStream_t>(stream));
}

spt_status spt_add(const spt_tensor* B, const spt_tensor* C, int32_t* out_pos, int32_t* out_crd0,
                   int32_t* out_crd1, int32_t* out_crd2, void* out_vals, int64_t* out_nnz_dev,
                   void* ws, size_t ws_bytes, void* stream) {
  return add_or_mul(0, B, C, out_pos, out_crd0, out_crd1, out_crd2, out_vals, out_nnz_dev, ws,
                    ws_bytes, stream);
}

spt_status spt_mul(const spt_tensor* B, const spt_tensor* C, int32_t* out_pos, int32_t* out_crd0,
                   int32_t* out_crd1, int32_t* out_crd2, void* out_vals, int64_t* out_nnz_dev,
                   void* ws, size_t ws_bytes, void* stream) {
  return add_or_mul(1, B, C, out_pos, out_crd0, out_crd1, out_crd2, out_vals, out_nnz_dev, ws,
                    ws_bytes, stream);
}

// A matrix in any composition the per-value reading is defined for.
static spt_status any_matrix(const spt_tensor* T, const char* what) {
  Format f = recognize(T);
  if (f == Format::Invalid) return SPT_ERR_INVALID_ARG;
  if (T->order != 2) return fail(SPT_ERR_UNSUPPORTED, "%s: operand must be a matrix", what);
  if (!generic_ok(T)) return SPT_ERR_UNSUPPORTED;
  return SPT_OK;
}

static int64_t dim_of(const spt_tensor* T, int mode) {
  for (int k = 0; k < T->nlevels; ++k)
    if (T->level[k].mode == mode) return T->level[k].N;
  return 0;
}

spt_status spt_mul_dense(const spt_tensor* B, const void* D, int64_t ld, void* out_vals, void* stream) {
  clear_error();
  spt_status st = any_matrix(B, "mul_dense");
  if (st != SPT_OK) return st;
  if (ld < dim_of(B, 1)) return fail(SPT_ERR_INVALID_ARG, "mul_dense: ld = %lld below the column count", (long long)ld);
  if (B->nvals > 0 && (!D || !out_vals)) return fail(SPT_ERR_INVALID_ARG, "mul_dense: D or out_vals is null");
  return mul_dense_dispatch(B, D, ld, out_vals, static_cast<hipStream_t>(stream));
}

spt_status spt_add_to_dense(const spt_tensor* B, const spt_tensor* C, void* A, int64_t ld, void* stream) {
  clear_error();
  spt_status st = any_matrix(B, "add_to_dense");
  if (st != SPT_OK) return st;
  st = any_matrix(C, "add_to_dense");
  if (st != SPT_OK) return st;
  if (B->dtype != C->dtype) return fail(SPT_ERR_INVALID_ARG, "add_to_dense: B and C differ in dtype");
  for (int m = 0; m < 2; ++m)
    if (dim_of(B, m) != dim_of(C, m))
      return fail(SPT_ERR_INVALID_ARG, "add_to_dense: dimension %d differs (%lld vs %lld)", m,
                  (long long)dim_of(B, m), (long long)dim_of(C, m));
  if (ld < dim_of(B, 1)) return fail(SPT_ERR_INVALID_ARG, "add_to_dense: ld = %lld below the column count", (long long)ld);
  if (!A && dim_of(B, 0) * dim_of(B, 1) > 0) return fail(SPT_ERR_INVALID_ARG, "add_to_dense: A is null");
  return add_to_dense_dispatch(B, C, A, ld, static_cast<hipStream_t>(stream));
}

size_t spt_add_workspace_bytes(const spt_tensor* B, const spt_tensor* C) {
  clear_error();
  Format fb, fc;
  if (add_operands(B, C, &fb, &fc) != SPT_OK) return 0;
  const size_t n = add_workspace(fb, fc, B, C);
  return n < 256 ? 256 : n;
}

size_t spt_workspace_bytes(int32_t op, const spt_tensor* T, int32_t J) {
  clear_error();
  Format f = recognize(T);
  if (f == Format::Invalid) return 0;
  if (f == Format::Unsupported || op == SPT_OP_TO_COO) {  // operations defined for any composition
    if (op == SPT_OP_SPMV && f == Format::Unsupported && is_aos_coo_matrix(T)) {
      clear_error();
      return aos_coo_spmv_workspace(T) + 256;
    }
    if (op == SPT_OP_SPMV && f == Format::Unsupported && (T->order == 2 || T->order == 4) &&
        generic_ok(T))
      return 256;
    if (op == SPT_OP_TO_COO && generic_ok(T)) return to_coo_workspace(T->nvals);
    if (g_err[0] == 0) fail(SPT_ERR_UNSUPPORTED, "operation %d is not defined for this composition", op);
    return 0;
  }
  size_t n = 0;
  switch (op) {
    case SPT_OP_SPMV_SPARSE_X:
      n = f == Format::CSR ? seg_spmv_workspace(T->nvals) : 0;
      break;
    case SPT_OP_SPDM:
      n = f == Format::COO2 ? mttkrp_workspace(f, T, J) : 0;
      break;
    case SPT_OP_SPMV:
      if (f == Format::CSR || (f == Format::COO2 && (T->level[0].flags & SPT_ORDERED)))
        n = seg_spmv_workspace(T->nvals);
      else if (f == Format::COO2)
        n = coo_unordered_workspace(T->dtype, T->nvals, T->level[0].N);
      else if (f == Format::BCSR && bcsr_fast_ok(T))
        n = bcsr_workspace(T);
      else if (f == Format::DCSR)
        n = dcsr_spmv_workspace(T);
      else if (f == Format::CSC)
        n = csc_spmv_workspace(T);
      break;
    case SPT_OP_COO_TO_CSR:
      n = f == Format::COO2 ? coo_to_csr_workspace(T) : 0;
      break;
    case SPT_OP_TTV:
      n = ttv_workspace(f, T);
      break;
    case SPT_OP_MTTKRP:
      n = mttkrp_workspace(f, T, J);
      break;
    case SPT_OP_TTM:
      n = (f == Format::COO3 || f == Format::CSF3) ? ttm_workspace(f, T, J) : 0;
      break;
    case SPT_OP_TO_CSF:
      n = f == Format::COO3 ? pack_csf_workspace(T->nvals) : 0;
      break;
    case SPT_OP_TO_ELL:
      n = (f == Format::COO2 || f == Format::CSR) ? pack_ell_workspace(f, T) : 0;
      break;
    case SPT_OP_DIA_OFFSETS:
      n = f == Format::COO2 ? dia_offsets_workspace(T) : 0;
      break;
    case SPT_OP_INNERPROD:
      n = (f == Format::COO3 || f == Format::COO2) ? innerprod_workspace(T->nvals) : 0;
      break;
    default:
      fail(SPT_ERR_INVALID_ARG, "unknown op %d", op);
      return 0;
  }
  return n < 256 ? 256 : n;
}

}  // extern "C"
