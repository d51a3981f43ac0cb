/*
 * oracle.c - plain CPU reference for the sparse tensor kernels (see oracle.h).
 * TEST INFRASTRUCTURE ONLY: slow on purpose, independent of the GPU library.
 *
 * Part 1 interprets the six level formats exactly as Table 2 of the paper
 * defines their level functions, and walks a tensor with the two iteration
 * templates of Figure 5 (coordinate value iteration for dense/range levels,
 * coordinate position iteration for the others).
 * Part 2 states each result (SpMV, COO->CSR, TTV, MTTKRP) by its definition
 * on top of that walk, accumulating in long double (fp64 data) or double
 * (fp32 data) and rounding once at the end.
 * Part 3 holds the plain per-format loop nests that the paper's generated
 * code amounts to (Section 5.2, 5.3); they are what the CPU baseline times.
 */
#include "oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Part 1: level functions (Table 2) and the hierarchy walk (Figure 5) */
/* ------------------------------------------------------------------ */

static int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }
static int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }

/* coord_bounds of dense and range levels. */
static void coord_bounds(const orc_level* L, int64_t i_parent, int64_t* lo,
                         int64_t* hi) {
  if (L->kind == ORC_DENSE) {
    *lo = 0;
    *hi = L->N;
  } else { /* range: bounds from offset[i_{k-1}] and the sizes N_k, M_k */
    int64_t off = L->offset[i_parent];
    *lo = imax(0, -off);
    *hi = imin(L->N, L->M - off);
  }
}

/* coord_access of dense and range levels: p_k = p_{k-1} * N_k + i_k. */
static int64_t coord_access(const orc_level* L, int64_t p_parent, int64_t i) {
  return p_parent * L->N + i;
}

/* pos_bounds of compressed / singleton / offset / hashed levels. */
static void pos_bounds(const orc_level* L, int64_t p_parent, int64_t* lo,
                       int64_t* hi) {
  switch (L->kind) {
    case ORC_COMPRESSED:
      *lo = L->pos[p_parent];
      *hi = L->pos[p_parent + 1];
      break;
    case ORC_HASHED:
      *lo = p_parent * L->M;
      *hi = (p_parent + 1) * L->M;
      break;
    default: /* singleton, offset: exactly the parent's position */
      *lo = p_parent;
      *hi = p_parent + 1;
  }
}

/* pos_access: coordinate stored at position p, and whether it is a child.
 * Singleton follows Table 2 except that a negative coordinate is read as
 * "unlabeled node" (ELL padding stored as -1), the same test the hashed level
 * applies to its empty buckets. */
/* Coordinate stored for position p: crd[p] for the struct-of-arrays layout; crd[p * stride]
 * for the array-of-structs variant of Section 5.2, where all levels of a component share one
 * interleaved array and each level starts at its own offset in it. */
static int64_t stored_crd(const orc_level* L, int64_t p) {
  return L->crd[L->crd_stride > 1 ? p * L->crd_stride : p];
}

static int pos_access(const orc_level* L, int64_t p, int64_t i_parent,
                      int64_t i_grand, int64_t* i_out) {
  switch (L->kind) {
    case ORC_COMPRESSED:
      *i_out = stored_crd(L, p);
      return 1;
    case ORC_SINGLETON:
      *i_out = stored_crd(L, p);
      return *i_out >= 0;
    case ORC_OFFSET: /* i_{k-1} + offset[i_{k-2}] */
      *i_out = i_parent + L->offset[i_grand];
      return 1;
    default: /* hashed */
      *i_out = stored_crd(L, p);
      return *i_out != -1;
  }
}

static int uses_coord_iteration(const orc_level* L) {
  return L->kind == ORC_DENSE || L->kind == ORC_RANGE;
}

int64_t orc_level_children(const orc_level* L, int64_t p_parent, int64_t i_parent,
                           int64_t i_grand, int64_t* out_i, int64_t* out_p,
                           int64_t cap) {
  int64_t n = 0, lo, hi;
  if (uses_coord_iteration(L)) {
    coord_bounds(L, i_parent, &lo, &hi);
    for (int64_t i = lo; i < hi; ++i) {
      if (n < cap) {
        out_i[n] = i;
        out_p[n] = coord_access(L, p_parent, i);
      }
      ++n;
    }
  } else {
    pos_bounds(L, p_parent, &lo, &hi);
    for (int64_t p = lo; p < hi; ++p) {
      int64_t i;
      if (pos_access(L, p, i_parent, i_grand, &i)) {
        if (n < cap) {
          out_i[n] = i;
          out_p[n] = p;
        }
        ++n;
      }
    }
  }
  return n;
}

int64_t orc_hashed_locate(const orc_level* L, int64_t p_parent, int64_t i,
                          int32_t* found) {
  int64_t W = L->M;
  int64_t p = i % W + p_parent * W;
  if (L->crd[p] != i && L->crd[p] != -1) {
    int64_t end = p;
    do {
      p = (p + 1) % W + p_parent * W;
    } while (L->crd[p] != i && L->crd[p] != -1 && p != end);
  }
  *found = (L->crd[p] == i);
  return p;
}

typedef struct {
  const orc_tensor* T;
  orc_visit_fn visit;
  void* ctx;
  int64_t lvl_coord[4];
} walk_state;

static void walk(walk_state* S, int k, int64_t p_parent) {
  const orc_tensor* T = S->T;
  if (k == T->nlevels) {
    int64_t coords[4] = {0, 0, 0, 0};
    for (int l = 0; l < T->nlevels; ++l)
      if (T->lvl[l].mode >= 0) coords[T->lvl[l].mode] = S->lvl_coord[l];
    S->visit(S->ctx, coords, p_parent);
    return;
  }
  const orc_level* L = &T->lvl[k];
  int64_t i_parent = k >= 1 ? S->lvl_coord[k - 1] : 0;
  int64_t i_grand = k >= 2 ? S->lvl_coord[k - 2] : 0;
  int64_t lo, hi;
  if (uses_coord_iteration(L)) {
    coord_bounds(L, i_parent, &lo, &hi);
    for (int64_t i = lo; i < hi; ++i) {
      S->lvl_coord[k] = i;
      walk(S, k + 1, coord_access(L, p_parent, i));
    }
  } else {
    pos_bounds(L, p_parent, &lo, &hi);
    for (int64_t p = lo; p < hi; ++p) {
      int64_t i;
      if (pos_access(L, p, i_parent, i_grand, &i)) {
        S->lvl_coord[k] = i;
        walk(S, k + 1, p);
      }
    }
  }
}

void orc_enumerate(const orc_tensor* T, orc_visit_fn visit, void* ctx) {
  walk_state S;
  S.T = T;
  S.visit = visit;
  S.ctx = ctx;
  memset(S.lvl_coord, 0, sizeof S.lvl_coord);
  walk(&S, 0, 0); /* one root parent at position 0 */
}

static double val_at(const orc_tensor* T, int64_t p) {
  return T->is_f64 ? ((const double*)T->vals)[p] : (double)((const float*)T->vals)[p];
}
static double dense_at(const void* a, int is_f64, int64_t n) {
  return is_f64 ? ((const double*)a)[n] : (double)((const float*)a)[n];
}

static void count_visit(void* ctx, const int64_t* c, int64_t p) {
  (void)c;
  (void)p;
  ++*(int64_t*)ctx;
}
int64_t orc_count(const orc_tensor* T) {
  int64_t n = 0;
  orc_enumerate(T, count_visit, &n);
  return n;
}

typedef struct {
  const orc_tensor* T;
  int64_t n, total;
  int64_t* coords;
  double* vals;
} dump_ctx;
static void dump_visit(void* vctx, const int64_t* c, int64_t p) {
  dump_ctx* D = (dump_ctx*)vctx;
  for (int m = 0; m < D->T->order; ++m) D->coords[m * D->total + D->n] = c[m];
  D->vals[D->n] = val_at(D->T, p);
  ++D->n;
}
void orc_to_coo(const orc_tensor* T, int64_t* coords_out, double* vals_out) {
  dump_ctx D = {T, 0, orc_count(T), coords_out, vals_out};
  orc_enumerate(T, dump_visit, &D);
}

/* ------------------------------------------------------------------ */
/* Part 2: results by definition                                       */
/* ------------------------------------------------------------------ */

typedef struct {
  const orc_tensor* T;
  const void* x;
  long double* acc;
  double* mag;
} spmv_ctx;
static void spmv_visit(void* vctx, const int64_t* c, int64_t p) {
  spmv_ctx* S = (spmv_ctx*)vctx;
  long double t = (long double)val_at(S->T, p) *
                  (long double)dense_at(S->x, S->T->is_f64, c[1]);
  S->acc[c[0]] += t;
  S->mag[c[0]] += fabs((double)t);
}
void orc_spmv(const orc_tensor* T, const void* x, int64_t rows, double* y,
              double* mag) {
  long double* acc = (long double*)calloc((size_t)(rows > 0 ? rows : 1), sizeof(long double));
  for (int64_t i = 0; i < rows; ++i) mag[i] = 0.0;
  spmv_ctx S = {T, x, acc, mag};
  orc_enumerate(T, spmv_visit, &S);
  for (int64_t i = 0; i < rows; ++i) y[i] = (double)acc[i];
  free(acc);
}

typedef struct {
  const orc_tensor* T;
  const void* x;
  long double* acc;
  double* mag;
  int64_t b1, b2;
} spmv_blk_ctx;
static void spmv_blk_visit(void* vctx, const int64_t* c, int64_t p) {
  spmv_blk_ctx* S = (spmv_blk_ctx*)vctx;
  /* component (i1, j1, i2, j2) of the 4th-order tensor is element (i1*b1 + i2, j1*b2 + j2) of the matrix */
  int64_t row = c[0] * S->b1 + c[2], col = c[1] * S->b2 + c[3];
  long double t = (long double)val_at(S->T, p) * (long double)dense_at(S->x, S->T->is_f64, col);
  S->acc[row] += t;
  S->mag[row] += fabs((double)t);
}
void orc_spmv_blocked(const orc_tensor* T, const void* x, int64_t b1, int64_t b2, int64_t rows,
                      double* y, double* mag) {
  long double* acc = (long double*)calloc((size_t)(rows > 0 ? rows : 1), sizeof(long double));
  for (int64_t i = 0; i < rows; ++i) mag[i] = 0.0;
  spmv_blk_ctx S = {T, x, acc, mag, b1, b2};
  orc_enumerate(T, spmv_blk_visit, &S);
  for (int64_t i = 0; i < rows; ++i) y[i] = (double)acc[i];
  free(acc);
}

typedef struct {
  const orc_tensor* T;
  const orc_tensor* X;
  long double* acc;
  double* mag;
} spmv_sx_ctx;
static void spmv_sx_visit(void* vctx, const int64_t* c, int64_t p) {
  spmv_sx_ctx* S = (spmv_sx_ctx*)vctx;
  const orc_level* L = &S->X->lvl[0];
  int64_t j = c[1], q = -1;
  if (L->kind == ORC_HASHED) {
    int32_t found = 0;
    q = orc_hashed_locate(L, 0, j, &found);
    if (!found) q = -1;
  } else { /* compressed: scan the parent's segment for coordinate j */
    for (int64_t r = L->pos[0]; r < L->pos[1]; ++r)
      if (L->crd[r] == j) {
        q = r;
        break;
      }
  }
  if (q < 0) return;
  long double t = (long double)val_at(S->T, p) * (long double)val_at(S->X, q);
  S->acc[c[0]] += t;
  S->mag[c[0]] += fabs((double)t);
}
void orc_spmv_sparse_x(const orc_tensor* T, const orc_tensor* X, int64_t rows, double* y,
                       double* mag) {
  long double* acc = (long double*)calloc((size_t)(rows > 0 ? rows : 1), sizeof(long double));
  for (int64_t i = 0; i < rows; ++i) mag[i] = 0.0;
  spmv_sx_ctx S = {T, X, acc, mag};
  orc_enumerate(T, spmv_sx_visit, &S);
  for (int64_t i = 0; i < rows; ++i) y[i] = (double)acc[i];
  free(acc);
}

typedef struct {
  const orc_tensor* T;
  const void* C;
  int32_t J;
  long double* acc;
  double* mag;
} spdm_ctx;
static void spdm_visit(void* vctx, const int64_t* co, int64_t p) {
  spdm_ctx* S = (spdm_ctx*)vctx;
  long double v = (long double)val_at(S->T, p);
  for (int32_t j = 0; j < S->J; ++j) {
    long double t = v * (long double)dense_at(S->C, S->T->is_f64, co[1] * S->J + j);
    S->acc[co[0] * S->J + j] += t;
    S->mag[co[0] * S->J + j] += fabs((double)t);
  }
}
void orc_spdm(const orc_tensor* B, const void* C, int32_t J, int64_t rows, double* A,
              double* mag) {
  int64_t n = rows * J;
  long double* acc = (long double*)calloc((size_t)(n > 0 ? n : 1), sizeof(long double));
  for (int64_t q = 0; q < n; ++q) mag[q] = 0.0;
  spdm_ctx S = {B, C, J, acc, mag};
  orc_enumerate(B, spdm_visit, &S);
  for (int64_t q = 0; q < n; ++q) A[q] = (double)acc[q];
  free(acc);
}

typedef struct {
  int64_t key;
  double val;
} kv_pair;
typedef struct {
  const orc_tensor* T;
  const int64_t* dims;
  kv_pair* out;
  int64_t n;
} lin_ctx;
static void lin_visit(void* vctx, const int64_t* co, int64_t p) {
  lin_ctx* S = (lin_ctx*)vctx;
  int64_t key = 0;
  for (int m = 0; m < S->T->order; ++m) key = key * S->dims[m] + co[m];
  S->out[S->n].key = key;
  S->out[S->n].val = val_at(S->T, p);
  ++S->n;
}
static int kv_cmp(const void* a, const void* b) {
  int64_t x = ((const kv_pair*)a)->key, y = ((const kv_pair*)b)->key;
  return x < y ? -1 : (x > y ? 1 : 0);
}
static kv_pair* linearise(const orc_tensor* T, const int64_t* dims, int64_t* n_out) {
  int64_t n = orc_count(T);
  kv_pair* a = (kv_pair*)malloc(sizeof(kv_pair) * (size_t)(n > 0 ? n : 1));
  lin_ctx S = {T, dims, a, 0};
  orc_enumerate(T, lin_visit, &S);
  qsort(a, (size_t)n, sizeof(kv_pair), kv_cmp);
  *n_out = n;
  return a;
}
double orc_innerprod(const orc_tensor* B, const orc_tensor* C, const int64_t* dims, double* mag) {
  long double space = 1.0L;
  for (int m = 0; m < B->order; ++m) space *= (long double)dims[m];
  *mag = 0.0;
  if (B->order != C->order || space >= 9.0e18L) return NAN;
  int64_t nb, nc;
  kv_pair* b = linearise(B, dims, &nb);
  kv_pair* c = linearise(C, dims, &nc);
  long double acc = 0.0L;
  int64_t pb = 0, pc = 0;
  while (pb < nb && pc < nc) { /* two-way merge: advance the smaller coordinate */
    if (b[pb].key < c[pc].key) ++pb;
    else if (b[pb].key > c[pc].key) ++pc;
    else {
      long double t = (long double)b[pb].val * (long double)c[pc].val;
      acc += t;
      *mag += fabs((double)t);
      ++pb;
      ++pc;
    }
  }
  free(b);
  free(c);
  return (double)acc;
}

static void emit_sum(int order, const int64_t* dims, int64_t key, double v, double mag,
                     int64_t n, int64_t cap, int32_t* const* out_crd, double* out_v,
                     double* out_mag) {
  if (n >= cap) return;
  for (int m = order - 1; m >= 0; --m) { /* undo the linearisation, last dimension first */
    out_crd[m][n] = (int32_t)(key % dims[m]);
    key /= dims[m];
  }
  out_v[n] = v;
  out_mag[n] = mag;
}
int64_t orc_add(const orc_tensor* B, const orc_tensor* C, const int64_t* dims, int64_t cap,
                int32_t* const* out_crd, double* out_v, double* out_mag) {
  long double space = 1.0L;
  for (int m = 0; m < B->order; ++m) space *= (long double)dims[m];
  if (B->order != C->order || space >= 9.0e18L) return -1;
  int64_t nb, nc;
  kv_pair* b = linearise(B, dims, &nb);
  kv_pair* c = linearise(C, dims, &nc);
  int64_t pb = 0, pc = 0, n = 0;
  while (pb < nb || pc < nc) { /* union: the smaller coordinate, or both when equal */
    if (pc >= nc || (pb < nb && b[pb].key < c[pc].key)) {
      emit_sum(B->order, dims, b[pb].key, b[pb].val, fabs(b[pb].val), n++, cap, out_crd, out_v,
               out_mag);
      ++pb;
    } else if (pb >= nb || c[pc].key < b[pb].key) {
      emit_sum(B->order, dims, c[pc].key, c[pc].val, fabs(c[pc].val), n++, cap, out_crd, out_v,
               out_mag);
      ++pc;
    } else {
      emit_sum(B->order, dims, b[pb].key, b[pb].val + c[pc].val,
               fabs(b[pb].val) + fabs(c[pc].val), n++, cap, out_crd, out_v, out_mag);
      ++pb;
      ++pc;
    }
  }
  free(b);
  free(c);
  return n;
}

typedef struct {
  const orc_tensor* T;
  const void* D;
  int64_t ld;
  double* out;
} muld_ctx;
static void muld_visit(void* vctx, const int64_t* c, int64_t p) {
  muld_ctx* S = (muld_ctx*)vctx;
  S->out[p] = val_at(S->T, p) * dense_at(S->D, S->T->is_f64, c[0] * S->ld + c[1]);
}
void orc_mul_dense(const orc_tensor* B, const void* D, int64_t ld, int64_t nvals, double* out) {
  for (int64_t p = 0; p < nvals; ++p) out[p] = 0.0; /* positions that hold no component */
  muld_ctx S = {B, D, ld, out};
  orc_enumerate(B, muld_visit, &S);
}

typedef struct {
  const orc_tensor* T;
  int64_t ld;
  double* A;
  double* mag;
} addd_ctx;
static void addd_visit(void* vctx, const int64_t* c, int64_t p) {
  addd_ctx* S = (addd_ctx*)vctx;
  double v = val_at(S->T, p);
  S->A[c[0] * S->ld + c[1]] += v; /* insert into the dense result: locate is i*ld + j */
  S->mag[c[0] * S->ld + c[1]] += fabs(v);
}
void orc_add_to_dense(const orc_tensor* B, const orc_tensor* C, int64_t rows, int64_t ld, double* A,
                      double* mag) {
  for (int64_t q = 0; q < rows * ld; ++q) A[q] = mag[q] = 0.0;
  addd_ctx S = {B, ld, A, mag};
  orc_enumerate(B, addd_visit, &S);
  S.T = C;
  orc_enumerate(C, addd_visit, &S);
}

int64_t orc_mul(const orc_tensor* B, const orc_tensor* C, const int64_t* dims, int64_t cap,
                int32_t* const* out_crd, double* out_v, double* out_mag) {
  long double space = 1.0L;
  for (int m = 0; m < B->order; ++m) space *= (long double)dims[m];
  if (B->order != C->order || space >= 9.0e18L) return -1;
  int64_t nb, nc;
  kv_pair* b = linearise(B, dims, &nb);
  kv_pair* c = linearise(C, dims, &nc);
  int64_t pb = 0, pc = 0, n = 0;
  while (pb < nb && pc < nc) { /* intersection: the loop ends with the first exhausted operand */
    int64_t ib = b[pb].key, ic = c[pc].key;
    int64_t i = ib < ic ? ib : ic; /* the coordinate visited in this step */
    if (ib == i && ic == i) {
      double v = b[pb].val * c[pc].val;
      emit_sum(B->order, dims, i, v, fabs(v), n++, cap, out_crd, out_v, out_mag);
    }
    if (ib == i) ++pb; /* each operand that holds the coordinate moves on */
    if (ic == i) ++pc;
  }
  free(b);
  free(c);
  return n;
}

int64_t orc_pack_csf(const orc_tensor* B, const int64_t* dims, int32_t* pos0, int32_t* crd0,
                     int32_t* pos1, int32_t* crd1, int32_t* pos2, int32_t* crd2, double* vals,
                     int64_t* counts) {
  long double space = (long double)dims[0] * (long double)dims[1] * (long double)dims[2];
  if (B->order != 3 || space >= 9.0e18L) return -1;
  int64_t n;
  kv_pair* e = linearise(B, dims, &n);
  int64_t n0 = 0, n1 = 0; /* entries appended to level 0 and level 1 so far */
  int64_t pi = -1, pj = -1;
  for (int64_t p = 0; p < n; ++p) {
    int64_t k = e[p].key % dims[2], j = (e[p].key / dims[2]) % dims[1],
            i = e[p].key / (dims[2] * dims[1]);
    int new_slice = p == 0 || i != pi;
    if (new_slice) {
      crd0[n0] = (int32_t)i; /* append_coord on level 0 */
      pos1[n0] = (int32_t)n1; /* its segment of level 1 starts here */
      ++n0;
    }
    if (new_slice || j != pj) {
      crd1[n1] = (int32_t)j;
      pos2[n1] = (int32_t)p;
      ++n1;
    }
    crd2[p] = (int32_t)k;
    vals[p] = e[p].val;
    pi = i;
    pj = j;
  }
  pos0[0] = 0;
  pos0[1] = (int32_t)n0; /* append_edges / append_finalize: each segment ends where the next starts */
  pos1[n0] = (int32_t)n1;
  pos2[n1] = (int32_t)n;
  counts[0] = n0;
  counts[1] = n1;
  free(e);
  return n;
}

int64_t orc_pack_hashed_rows(const orc_tensor* A, const int64_t* dims, int64_t W, int32_t* crd,
                             double* vals) {
  int64_t N = dims[0], M = dims[1], n, dropped = 0;
  for (int64_t q = 0; q < N * W; ++q) { /* insert_init */
    crd[q] = -1;
    vals[q] = 0.0;
  }
  orc_level H = {0};
  H.kind = ORC_HASHED;
  H.N = M;
  H.M = W;
  H.crd = crd;
  kv_pair* e = linearise(A, dims, &n);
  for (int64_t p = 0; p < n; ++p) {
    int64_t i = e[p].key / M, j = e[p].key % M;
    int32_t found;
    int64_t slot = orc_hashed_locate(&H, i, j, &found); /* locate, then insert_coord */
    if (found || crd[slot] == -1) {
      crd[slot] = (int32_t)j;
      vals[slot] = e[p].val;
    } else {
      ++dropped;
    }
  }
  free(e);
  return dropped;
}

int64_t orc_pack_ell(const orc_tensor* A, const int64_t* dims, int64_t W, int32_t* crd,
                     double* vals) {
  int64_t N = dims[0], M = dims[1], n;
  for (int64_t q = 0; q < W * N; ++q) {
    crd[q] = -1;
    vals[q] = 0.0;
  }
  kv_pair* e = linearise(A, dims, &n);
  int64_t longest = 0, row = -1, k = 0;
  for (int64_t p = 0; p < n; ++p) {
    int64_t i = e[p].key / M, j = e[p].key % M;
    k = i == row ? k + 1 : 0; /* slot = rank of the entry inside its row */
    row = i;
    if (k < W) {
      crd[k * N + i] = (int32_t)j;
      vals[k * N + i] = e[p].val;
    }
    if (k + 1 > longest) longest = k + 1;
  }
  free(e);
  return longest;
}

static int i64_cmp(const void* a, const void* b) {
  int64_t x = *(const int64_t*)a, y = *(const int64_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}
int64_t orc_dia_offsets(const orc_tensor* A, const int64_t* dims, int64_t cap, int32_t* offsets) {
  int64_t M = dims[1], n;
  kv_pair* e = linearise(A, dims, &n);
  int64_t* d = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
  for (int64_t p = 0; p < n; ++p) d[p] = e[p].key % M - e[p].key / M;
  qsort(d, (size_t)n, sizeof(int64_t), i64_cmp);
  int64_t K = 0;
  for (int64_t p = 0; p < n; ++p)
    if (p == 0 || d[p] != d[p - 1]) {
      if (K < cap) offsets[K] = (int32_t)d[p];
      ++K;
    }
  free(d);
  free(e);
  return K;
}
void orc_pack_dia(const orc_tensor* A, const int64_t* dims, int64_t K, const int32_t* offsets,
                  double* vals) {
  int64_t N = dims[0], M = dims[1], n;
  for (int64_t q = 0; q < K * N; ++q) vals[q] = 0.0;
  kv_pair* e = linearise(A, dims, &n);
  for (int64_t p = 0; p < n; ++p) {
    int64_t i = e[p].key / M, j = e[p].key % M;
    for (int64_t d = 0; d < K; ++d) /* locate the diagonal, then insert */
      if (offsets[d] == j - i) vals[d * N + i] = e[p].val;
  }
  free(e);
}

/* Stable bottom-up merge sort of an index permutation by one or two int32 keys. */
static int key_less(const int32_t* k0, const int32_t* k1, int64_t a, int64_t b) {
  if (k0[a] != k0[b]) return k0[a] < k0[b];
  if (k1 && k1[a] != k1[b]) return k1[a] < k1[b];
  return 0;
}
static void stable_sort_perm(int64_t n, int64_t* perm, const int32_t* k0,
                             const int32_t* k1) {
  int64_t* tmp = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
  int64_t* src = perm;
  int64_t* dst = tmp;
  for (int64_t w = 1; w < n; w *= 2) {
    for (int64_t lo = 0; lo < n; lo += 2 * w) {
      int64_t mid = imin(lo + w, n), hi = imin(lo + 2 * w, n);
      int64_t a = lo, b = mid, o = lo;
      while (a < mid && b < hi) {
        /* take from the right run only if strictly smaller: stability */
        if (key_less(k0, k1, src[b], src[a])) dst[o++] = src[b++];
        else dst[o++] = src[a++];
      }
      while (a < mid) dst[o++] = src[a++];
      while (b < hi) dst[o++] = src[b++];
    }
    int64_t* t = src;
    src = dst;
    dst = t;
  }
  if (src != perm) memcpy(perm, src, sizeof(int64_t) * (size_t)n);
  free(tmp);
}

void orc_coo_to_csr(int64_t nnz, int64_t nrows, const int32_t* row,
                    const int32_t* col, const void* vals, int32_t esize,
                    int32_t order, int32_t* pos_out, int32_t* crd_out,
                    void* vals_out, int64_t* perm_out) {
  int64_t* perm = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
  for (int64_t n = 0; n < nnz; ++n) perm[n] = n;
  stable_sort_perm(nnz, perm, row, order == 0 ? col : NULL);
  /* Assemble the compressed column level with Table 3's append functions. */
  for (int64_t p = 0; p <= nrows; ++p) pos_out[p] = 0; /* append_init */
  int64_t q = 0;
  for (int64_t i = 0; i < nrows; ++i) {
    int64_t pbegin = q;
    while (q < nnz && row[perm[q]] == i) {
      crd_out[q] = col[perm[q]]; /* append_coord */
      memcpy((char*)vals_out + q * esize, (const char*)vals + perm[q] * esize,
             (size_t)esize);
      ++q;
    }
    pos_out[i + 1] = (int32_t)(q - pbegin); /* append_edges */
  }
  int64_t cumsum = pos_out[0]; /* append_finalize */
  for (int64_t p = 1; p <= nrows; ++p) {
    cumsum += pos_out[p];
    pos_out[p] = (int32_t)cumsum;
  }
  if (perm_out) memcpy(perm_out, perm, sizeof(int64_t) * (size_t)nnz);
  free(perm);
}

typedef struct {
  const orc_tensor* T;
  const void* c;
  int64_t n;
  int32_t *ki, *kj;
  long double* term;
} ttv_ctx;
static void ttv_visit(void* vctx, const int64_t* co, int64_t p) {
  ttv_ctx* S = (ttv_ctx*)vctx;
  S->ki[S->n] = (int32_t)co[0];
  S->kj[S->n] = (int32_t)co[1];
  S->term[S->n] = (long double)val_at(S->T, p) *
                  (long double)dense_at(S->c, S->T->is_f64, co[2]);
  ++S->n;
}
int64_t orc_ttv(const orc_tensor* B, const void* c, int64_t cap, int32_t* out_i,
                int32_t* out_j, double* out_v, double* out_mag) {
  int64_t total = orc_count(B);
  size_t a = (size_t)(total > 0 ? total : 1);
  ttv_ctx S = {B, c, 0, (int32_t*)malloc(4 * a), (int32_t*)malloc(4 * a),
               (long double*)malloc(sizeof(long double) * a)};
  orc_enumerate(B, ttv_visit, &S);
  int64_t* perm = (int64_t*)malloc(sizeof(int64_t) * a);
  for (int64_t n = 0; n < total; ++n) perm[n] = n;
  stable_sort_perm(total, perm, S.ki, S.kj);
  int64_t nout = 0;
  int64_t n = 0;
  while (n < total) {
    int32_t i = S.ki[perm[n]], j = S.kj[perm[n]];
    long double acc = 0.0L;
    double mag = 0.0;
    while (n < total && S.ki[perm[n]] == i && S.kj[perm[n]] == j) {
      acc += S.term[perm[n]];
      mag += fabs((double)S.term[perm[n]]);
      ++n;
    }
    if (nout < cap) {
      out_i[nout] = i;
      out_j[nout] = j;
      out_v[nout] = (double)acc;
      out_mag[nout] = mag;
    }
    ++nout;
  }
  free(perm);
  free(S.ki);
  free(S.kj);
  free(S.term);
  return nout;
}

typedef struct {
  int64_t n;
  int32_t *ki, *kj, *kl;
  int64_t* leaf;
} ttm_ctx;
static void ttm_visit(void* vctx, const int64_t* co, int64_t p) {
  ttm_ctx* S = (ttm_ctx*)vctx;
  S->ki[S->n] = (int32_t)co[0];
  S->kj[S->n] = (int32_t)co[1];
  S->kl[S->n] = (int32_t)co[2];
  S->leaf[S->n] = p;
  ++S->n;
}
int64_t orc_ttm(const orc_tensor* B, const void* C, int32_t K, int64_t L, int64_t cap,
                int32_t* out_i, int32_t* out_j, double* out_v, double* out_mag) {
  int64_t total = orc_count(B);
  size_t a = (size_t)(total > 0 ? total : 1);
  ttm_ctx S = {0, (int32_t*)malloc(4 * a), (int32_t*)malloc(4 * a), (int32_t*)malloc(4 * a),
               (int64_t*)malloc(8 * a)};
  orc_enumerate(B, ttm_visit, &S);
  int64_t* perm = (int64_t*)malloc(sizeof(int64_t) * a);
  for (int64_t n = 0; n < total; ++n) perm[n] = n;
  stable_sort_perm(total, perm, S.ki, S.kj);
  int f = B->is_f64;
  int64_t nout = 0, n = 0;
  while (n < total) {
    int32_t i = S.ki[perm[n]], j = S.kj[perm[n]];
    int64_t first = n;
    while (n < total && S.ki[perm[n]] == i && S.kj[perm[n]] == j) ++n;
    if (nout < cap) {
      out_i[nout] = i;
      out_j[nout] = j;
      for (int32_t k = 0; k < K; ++k) { /* A_ijk = sum over the fibre's l of B_ijl C_kl */
        long double sum = 0.0L;
        double mag = 0.0;
        for (int64_t q = first; q < n; ++q) {
          long double t = (long double)val_at(B, S.leaf[perm[q]]) *
                          (long double)dense_at(C, f, (int64_t)k * L + S.kl[perm[q]]);
          sum += t;
          mag += fabs((double)t);
        }
        out_v[nout * K + k] = (double)sum;
        out_mag[nout * K + k] = mag;
      }
    }
    ++nout;
  }
  free(perm);
  free(S.ki);
  free(S.kj);
  free(S.kl);
  free(S.leaf);
  return nout;
}

typedef struct {
  const orc_tensor* T;
  const void *C, *D;
  int32_t J;
  long double* acc;
  double* mag;
} mttkrp_ctx;
static void mttkrp_visit(void* vctx, const int64_t* co, int64_t p) {
  mttkrp_ctx* S = (mttkrp_ctx*)vctx;
  int f = S->T->is_f64;
  long double v = (long double)val_at(S->T, p);
  for (int32_t j = 0; j < S->J; ++j) {
    long double t = v * (long double)dense_at(S->C, f, co[1] * S->J + j) *
                    (long double)dense_at(S->D, f, co[2] * S->J + j);
    S->acc[co[0] * S->J + j] += t;
    S->mag[co[0] * S->J + j] += fabs((double)t);
  }
}
void orc_mttkrp(const orc_tensor* B, const void* C, const void* D, int32_t J,
                int64_t dim0, double* A, double* mag) {
  int64_t n = dim0 * J;
  long double* acc = (long double*)calloc((size_t)(n > 0 ? n : 1), sizeof(long double));
  for (int64_t q = 0; q < n; ++q) mag[q] = 0.0;
  mttkrp_ctx S = {B, C, D, J, acc, mag};
  orc_enumerate(B, mttkrp_visit, &S);
  for (int64_t q = 0; q < n; ++q) A[q] = (double)acc[q];
  free(acc);
}

/* ------------------------------------------------------------------ */
/* Part 3: plain loop nests per format, native dtype                   */
/* ------------------------------------------------------------------ */

/* The loops whose iterations write disjoint outputs (rows, fibres, slices) carry an OpenMP
 * pragma that takes effect only in the build with -fopenmp (the all-cores leg of the CPU
 * baseline); each iteration's arithmetic and its order of additions are the same either
 * way. The scatter loops (COO SpMV, COO MTTKRP, COO TTV's append) stay serial: the paper's
 * generated code is a single loop over the stored entries there. */
#ifdef _OPENMP
#include <omp.h>
#define ORC_PARALLEL_FOR _Pragma("omp parallel for schedule(static)")
int32_t orc_set_threads(int32_t n) {
  if (n > 0) omp_set_num_threads(n);
  return omp_get_max_threads();
}
#else
#define ORC_PARALLEL_FOR
int32_t orc_set_threads(int32_t n) {
  (void)n;
  return 1;
}
#endif

#define PLAIN_SPMV_CSR(TY)                                              \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* xv = (const TY*)x;                                        \
    TY* yv = (TY*)y;                                                    \
    ORC_PARALLEL_FOR                                                    \
    for (int64_t i = 0; i < N; ++i) {                                   \
      TY s = 0;                                                         \
      for (int32_t p = pos[i]; p < pos[i + 1]; ++p) s += v[p] * xv[crd[p]]; \
      yv[i] = s;                                                        \
    }                                                                   \
  }
void orc_plain_spmv_csr(int64_t N, const int32_t* pos, const int32_t* crd,
                        const void* vals, const void* x, void* y, int32_t is_f64) {
  if (is_f64) PLAIN_SPMV_CSR(double) else PLAIN_SPMV_CSR(float)
}

#define PLAIN_SPMV_COO(TY)                                              \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* xv = (const TY*)x;                                        \
    TY* yv = (TY*)y;                                                    \
    for (int64_t i = 0; i < N; ++i) yv[i] = 0;                          \
    for (int64_t p = 0; p < nnz; ++p) yv[row[p]] += v[p] * xv[col[p]];  \
  }
void orc_plain_spmv_coo(int64_t N, int64_t nnz, const int32_t* row,
                        const int32_t* col, const void* vals, const void* x,
                        void* y, int32_t is_f64) {
  if (is_f64) PLAIN_SPMV_COO(double) else PLAIN_SPMV_COO(float)
}

#define PLAIN_SPMV_DIA(TY)                                              \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* xv = (const TY*)x;                                        \
    TY* yv = (TY*)y;                                                    \
    for (int64_t i = 0; i < N; ++i) yv[i] = 0;                          \
    for (int64_t d = 0; d < K; ++d) {                                   \
      int64_t off = offset[d];                                          \
      int64_t lo = imax(0, -off), hi = imin(N, M - off);                \
      ORC_PARALLEL_FOR                                                  \
      for (int64_t i = lo; i < hi; ++i) yv[i] += v[d * N + i] * xv[i + off]; \
    }                                                                   \
  }
void orc_plain_spmv_dia(int64_t N, int64_t M, int64_t K, const int32_t* offset,
                        const void* vals, const void* x, void* y, int32_t is_f64) {
  if (is_f64) PLAIN_SPMV_DIA(double) else PLAIN_SPMV_DIA(float)
}

#define PLAIN_SPMV_ELL(TY)                                              \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* xv = (const TY*)x;                                        \
    TY* yv = (TY*)y;                                                    \
    for (int64_t i = 0; i < N; ++i) yv[i] = 0;                          \
    for (int64_t k = 0; k < W; ++k) {                                   \
      ORC_PARALLEL_FOR                                                  \
      for (int64_t i = 0; i < N; ++i) {                                 \
        int32_t j = crd[k * N + i];                                     \
        if (j >= 0) yv[i] += v[k * N + i] * xv[j];                      \
      }                                                                 \
    }                                                                   \
  }
void orc_plain_spmv_ell(int64_t N, int64_t W, const int32_t* crd,
                        const void* vals, const void* x, void* y, int32_t is_f64) {
  if (is_f64) PLAIN_SPMV_ELL(double) else PLAIN_SPMV_ELL(float)
}

#define PLAIN_TTV_COO(TY)                                               \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* cv = (const TY*)c;                                        \
    TY* ov = (TY*)out_v;                                                \
    int64_t p = 0;                                                      \
    while (p < nnz) {                                                   \
      int32_t i = ci[p], j = cj[p];                                     \
      TY s = 0;                                                         \
      while (p < nnz && ci[p] == i && cj[p] == j) {                     \
        s += v[p] * cv[ck[p]];                                          \
        ++p;                                                            \
      }                                                                 \
      out_i[nout] = i;                                                  \
      out_j[nout] = j;                                                  \
      ov[nout] = s;                                                     \
      ++nout;                                                           \
    }                                                                   \
  }
int64_t orc_plain_ttv_coo(int64_t nnz, const int32_t* ci, const int32_t* cj,
                          const int32_t* ck, const void* vals, const void* c,
                          int32_t* out_i, int32_t* out_j, void* out_v,
                          int32_t is_f64) {
  int64_t nout = 0;
  if (is_f64) PLAIN_TTV_COO(double) else PLAIN_TTV_COO(float)
  return nout;
}

#define PLAIN_TTV_CSF(TY)                                               \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* cv = (const TY*)c;                                        \
    TY* ov = (TY*)out_v;                                                \
    ORC_PARALLEL_FOR                                                    \
    for (int64_t f = 0; f < nfib; ++f) {                                \
      TY s = 0;                                                         \
      for (int32_t p = pos2[f]; p < pos2[f + 1]; ++p) s += v[p] * cv[crd2[p]]; \
      ov[f] = s;                                                        \
    }                                                                   \
  }
void orc_plain_ttv_csf(int64_t nfib, const int32_t* pos2, const int32_t* crd2,
                       const void* vals, const void* c, void* out_v,
                       int32_t is_f64) {
  if (is_f64) PLAIN_TTV_CSF(double) else PLAIN_TTV_CSF(float)
}

#define PLAIN_MTTKRP_COO(TY)                                            \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* Cv = (const TY*)C;                                        \
    const TY* Dv = (const TY*)D;                                        \
    TY* Av = (TY*)A;                                                    \
    for (int64_t q = 0; q < dim0 * J; ++q) Av[q] = 0;                   \
    for (int64_t p = 0; p < nnz; ++p) {                                 \
      const TY* cr = Cv + (int64_t)ck[p] * J;                           \
      const TY* dr = Dv + (int64_t)cl[p] * J;                           \
      TY* ar = Av + (int64_t)ci[p] * J;                                 \
      for (int32_t j = 0; j < J; ++j) ar[j] += v[p] * cr[j] * dr[j];    \
    }                                                                   \
  }
void orc_plain_mttkrp_coo(int64_t nnz, int64_t dim0, const int32_t* ci,
                          const int32_t* ck, const int32_t* cl, const void* vals,
                          const void* C, const void* D, int32_t J, void* A,
                          int32_t is_f64) {
  if (is_f64) PLAIN_MTTKRP_COO(double) else PLAIN_MTTKRP_COO(float)
}

#define PLAIN_MTTKRP_CSF(TY)                                            \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* Cv = (const TY*)C;                                        \
    const TY* Dv = (const TY*)D;                                        \
    TY* Av = (TY*)A;                                                    \
    for (int64_t q = 0; q < dim0 * J; ++q) Av[q] = 0;                   \
    ORC_PARALLEL_FOR                                                    \
    for (int32_t p0 = pos0[0]; p0 < pos0[1]; ++p0) {                    \
      TY t[1024]; /* J <= 1024 */                                       \
      TY* ar = Av + (int64_t)crd0[p0] * J;                              \
      for (int32_t p1 = pos1[p0]; p1 < pos1[p0 + 1]; ++p1) {            \
        const TY* cr = Cv + (int64_t)crd1[p1] * J;                      \
        for (int32_t j = 0; j < J; ++j) t[j] = 0;                       \
        for (int32_t p2 = pos2[p1]; p2 < pos2[p1 + 1]; ++p2) {          \
          const TY* dr = Dv + (int64_t)crd2[p2] * J;                    \
          for (int32_t j = 0; j < J; ++j) t[j] += v[p2] * dr[j];        \
        }                                                               \
        for (int32_t j = 0; j < J; ++j) ar[j] += cr[j] * t[j];          \
      }                                                                 \
    }                                                                   \
  }
void orc_plain_mttkrp_csf(int64_t dim0, const int32_t* pos0, const int32_t* crd0,
                          const int32_t* pos1, const int32_t* crd1,
                          const int32_t* pos2, const int32_t* crd2,
                          const void* vals, const void* C, const void* D,
                          int32_t J, void* A, int32_t is_f64) {
  if (is_f64) PLAIN_MTTKRP_CSF(double) else PLAIN_MTTKRP_CSF(float)
}

#define PLAIN_SPDM_COO(TY)                                              \
  {                                                                     \
    const TY* v = (const TY*)vals;                                      \
    const TY* Cv = (const TY*)C;                                        \
    TY* Av = (TY*)A;                                                    \
    for (int64_t q = 0; q < rows * J; ++q) Av[q] = 0;                   \
    for (int64_t p = 0; p < nnz; ++p) {                                 \
      const TY* cr = Cv + (int64_t)col[p] * J;                          \
      TY* ar = Av + (int64_t)row[p] * J;                                \
      for (int32_t j = 0; j < J; ++j) ar[j] += v[p] * cr[j];            \
    }                                                                   \
  }
void orc_plain_spdm_coo(int64_t nnz, int64_t rows, const int32_t* row, const int32_t* col,
                        const void* vals, const void* C, int32_t J, void* A, int32_t is_f64) {
  if (is_f64) PLAIN_SPDM_COO(double) else PLAIN_SPDM_COO(float)
}
