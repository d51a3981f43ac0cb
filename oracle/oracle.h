/*
 * oracle.h - CPU reference ("oracle") for sparse tensor kernels over the
 * coordinate-hierarchy level formats of the paper (Section 3, Table 2, Table 3).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE. It is deliberately plain and
 * slow: a literal interpreter of the level functions plus the textbook
 * definition of each result, accumulated in extended precision. It shares no
 * code, header or table with the GPU library; only tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it.
 *
 * All pointers are HOST pointers. Index arrays are int32. Values are float
 * (is_f64 = 0) or double (is_f64 = 1); reference results are always returned
 * as double, together with the magnitude sum |term| that scales the tolerance.
 */
#ifndef ORACLE_H
#define ORACLE_H
#include <stdint.h>

enum { ORC_DENSE = 0, ORC_COMPRESSED = 1, ORC_SINGLETON = 2, ORC_RANGE = 3,
       ORC_OFFSET = 4, ORC_HASHED = 5 };

typedef struct {
  int32_t kind;   /* ORC_* */
  int32_t mode;   /* tensor dimension encoded by this level, -1 if none */
  int64_t N;      /* dense/range: N_k; others: dimension size */
  int64_t M;      /* range: M_k; hashed: W_k */
  const int32_t* pos;
  const int32_t* crd;
  const int32_t* offset;
  int64_t crd_stride; /* elements between the coordinates of consecutive positions; 0 or 1 =
                         contiguous; > 1 = interleaved (array-of-structs COO, Section 5.2),
                         honoured by the level walk (orc_enumerate and what builds on it) */
} orc_level;

typedef struct {
  int32_t order;    /* tensor dimensions */
  int32_t nlevels;  /* levels */
  int32_t is_f64;
  int32_t pad;
  orc_level lvl[4];
  const void* vals;
} orc_tensor;

/* Visitor: coords[m] = coordinate along tensor dimension m, p = leaf position. */
typedef void (*orc_visit_fn)(void* ctx, const int64_t* coords, int64_t p);

/* Walk every stored leaf of T in storage order (Figure 5 iteration templates
 * applied level by level with the level functions of Table 2). */
void orc_enumerate(const orc_tensor* T, orc_visit_fn visit, void* ctx);

/* Children of one parent in one level: Table 2 for that level kind.
 * p_parent: parent position; i_parent: parent coordinate; i_grand: coordinate
 * two levels up (the offset level reads offset[i_grand], Table 2).
 * Writes up to cap (coordinate, position) pairs; returns the child count. */
int64_t orc_level_children(const orc_level* L, int64_t p_parent, int64_t i_parent,
                           int64_t i_grand, int64_t* out_i, int64_t* out_p,
                           int64_t cap);

/* Hashed level locate (Table 2): returns position, *found set to 0/1. */
int64_t orc_hashed_locate(const orc_level* L, int64_t p_parent, int64_t i,
                          int32_t* found);

/* Number of stored leaves. */
int64_t orc_count(const orc_tensor* T);
/* Dump to coordinate lists: coords_out[m*count + n], vals_out[n] (as double). */
void orc_to_coo(const orc_tensor* T, int64_t* coords_out, double* vals_out);

/* y_i = sum over stored (i,j): v * x_j (Section 5.2). rows = len(y).
 * y and mag (sum of |v*x_j|) are overwritten. x has the dtype of T. */
void orc_spmv(const orc_tensor* T, const void* x, int64_t rows, double* y,
              double* mag);

/* SpMV on a blocked matrix format cast as a 4th-order tensor (Section 3.2: BCSR, CSB): T has
 * dimensions (block rows, block columns, b1 rows per block, b2 columns per block) in any legal
 * composition of levels, and component (i1, j1, i2, j2) is matrix element (i1*b1 + i2,
 * j1*b2 + j2): y(i1, i2) = sum over stored components of A(i1, j1, i2, j2) x(j1, j2), with y and
 * x stored flat. rows = len(y) = block rows * b1. y and mag are overwritten. */
void orc_spmv_blocked(const orc_tensor* T, const void* x, int64_t b1, int64_t b2, int64_t rows,
                      double* y, double* mag);

/* y = A x with x stored as a 1st-order tensor X (Section 5.4, Figure 16):
 * one compressed level (sparse vector) or one hashed level (hash map). Every
 * stored (i,j) of A looks x_j up in X: by the hashed level's locate function
 * (Table 2), or, for the compressed level, in the list of X's stored
 * coordinates (absent = 0). */
void orc_spmv_sparse_x(const orc_tensor* T, const orc_tensor* X, int64_t rows, double* y,
                       double* mag);

/* SpDM A = B C (Section 5.2, Figure 11): B any matrix format, C dense cols x J
 * row-major in B's dtype; A, mag: rows x J. */
void orc_spdm(const orc_tensor* B, const void* C, int32_t J, int64_t rows, double* A,
              double* mag);

/* INNERPROD alpha = sum_ijk B_ijk C_ijk (Section 5.3) of two tensors of equal order and
 * dimensions dims[order], in any formats: both are walked, ordered by linearised coordinate,
 * and co-iterated with the two-way merge of Section 4.4 (coordinates are assumed unique in
 * each operand). Returns alpha; *mag receives sum |B C|. Returns NaN if the linearised
 * coordinate would overflow 63 bits. */
double orc_innerprod(const orc_tensor* B, const orc_tensor* C, const int64_t* dims, double* mag);

/* A = B + C with a sparse result (Section 5.2 matrix addition, Section 5.3 PLUS): the union
 * merge of Section 4.4 over both operands ordered by linearised coordinate; a coordinate
 * stored in both gives one entry holding the sum, a coordinate stored in one gives that entry
 * (results that cancel to zero stay stored). Coordinates are assumed unique per operand.
 * out_crd: order arrays of capacity cap each (out_crd[m][n] = coordinate m of entry n),
 * out_v / out_mag (|b| + |c|) capacity cap. Returns the entry count (-1: 63-bit overflow of
 * the linearised coordinate or operands of different order). */
int64_t orc_add(const orc_tensor* B, const orc_tensor* C, const int64_t* dims, int64_t cap,
                int32_t* const* out_crd, double* out_v, double* out_mag);

/* A = B .* D with D a dense N x M matrix (row-major, leading dimension ld), the first of the
 * element-wise products of Figure 1: the result has B's structure, so only its values are
 * produced, out[p] = B.vals[p] * D(i, j) for the component (i, j) at leaf position p, 0 at
 * positions that hold no component (ELL padding, cells outside a range level). D has B's dtype.
 * out: nvals doubles. B: any composition that stores a matrix. */
void orc_mul_dense(const orc_tensor* B, const void* D, int64_t ld, int64_t nvals, double* out);

/* A = B + C with a dense result (the CSR + COO example of Section 4.4, Figure 9): a dense
 * output supports insert (Table 3), so no merge is needed: each operand is walked on its own
 * and every component is added at A[i*ld + j]. A and mag (sum of |terms|): rows*ld doubles,
 * overwritten. B, C: any compositions that store matrices of equal dimensions. */
void orc_add_to_dense(const orc_tensor* B, const orc_tensor* C, int64_t rows, int64_t ld, double* A,
                      double* mag);

/* A = B .* C (element-wise product) with a sparse result: the intersection merge of Section 4.4
 * (the running example of Sections 1 and 4, Figure 1): both operands are walked in order of
 * linearised coordinate, the one with the smaller coordinate advances, and only a coordinate
 * stored in both produces an entry (the product; products that are zero stay stored).
 * Arguments and return as orc_add; out_mag = |b * c|. */
int64_t orc_mul(const orc_tensor* B, const orc_tensor* C, const int64_t* dims, int64_t cap,
                int32_t* const* out_crd, double* out_v, double* out_mag);

/* Packing a tensor (any format) into CSF, ELL or DIA, Section 3.4: the entries are walked,
 * ordered by linearised coordinate, and appended (CSF, ELL) or inserted (DIA) into the
 * target's levels. Values are returned as double (exact for fp32 and fp64 sources).
 *
 * orc_pack_csf, 3rd order: level k has pos_k and crd_k (pos0 has 2 entries); a coordinate is
 * appended to level 0 / 1 when it differs from the previous entry's (i) / (i,j), every entry
 * appends its k to level 2; append_edges closes a parent's segment, so pos holds running
 * sums. counts[0], counts[1] = slices, fibres. Arrays need capacity nnz (+1 for pos).
 * Returns nnz, or -1 on overflow of the linearised coordinate.
 *
 * orc_pack_ell: cell (k, i) at k*N + i holds the k-th stored entry of row i (columns
 * ascending); unused cells have crd -1 and value 0. Rows longer than W lose their tail.
 * Returns the longest row.
 *
 * orc_dia_offsets: the distinct values of col - row, ascending (at most cap are written);
 * returns their number K. orc_pack_dia: cell (d, i) at d*N + i = the entry of row i on
 * diagonal offsets[d], zero where none is stored (coordinates unique). */
/* orc_pack_hashed_rows: the matrix as (dense rows, hashed columns of width W), assembled with
 * Table 3's insert functions: insert_init fills crd with -1; every entry (walked in order of
 * linearised coordinate) is inserted at the position the hashed level's locate returns (first
 * slot at or after j % W, wrapping, that holds j or is empty). Returns the number of entries
 * that found their row's table full. */
int64_t orc_pack_hashed_rows(const orc_tensor* A, const int64_t* dims, int64_t W, int32_t* crd,
                             double* vals);

int64_t orc_pack_csf(const orc_tensor* B, const int64_t* dims, int32_t* pos0, int32_t* crd0,
                     int32_t* pos1, int32_t* crd1, int32_t* pos2, int32_t* crd2, double* vals,
                     int64_t* counts);
int64_t orc_pack_ell(const orc_tensor* A, const int64_t* dims, int64_t W, int32_t* crd,
                     double* vals);
int64_t orc_dia_offsets(const orc_tensor* A, const int64_t* dims, int64_t cap, int32_t* offsets);
void orc_pack_dia(const orc_tensor* A, const int64_t* dims, int64_t K, const int32_t* offsets,
                  double* vals);

/* COO -> CSR index assembly. order 0: by (row,col), ties keep input order;
 * order 1: by row, input order kept inside a row. pos via Table 3's
 * append_init / append_edges / append_finalize. perm_out[n] = input index of
 * output entry n (may be NULL). esize = bytes per value (4 or 8). */
void orc_coo_to_csr(int64_t nnz, int64_t nrows, const int32_t* row,
                    const int32_t* col, const void* vals, int32_t esize,
                    int32_t order, int32_t* pos_out, int32_t* crd_out,
                    void* vals_out, int64_t* perm_out);

/* TTM A_ijk = sum_l B_ijl C_kl (Section 5.3), C dense K x L row-major. One output fibre per
 * distinct (i,j) holding a stored entry, ascending (i,j); fibre f holds K values
 * out_v[f*K .. f*K+K) (and magnitudes sum |B C|). Returns the fibre count; outputs have
 * capacity cap fibres. */
int64_t orc_ttm(const orc_tensor* B, const void* C, int32_t K, int64_t L, int64_t cap,
                int32_t* out_i, int32_t* out_j, double* out_v, double* out_mag);

/* TTV A_ij = sum_k B_ijk c_k (Section 5.3): one output entry per distinct
 * (i,j) holding a stored entry, ascending (i,j). Returns the entry count;
 * outputs have capacity cap (= number of leaves is always enough). */
int64_t orc_ttv(const orc_tensor* B, const void* c, int64_t cap, int32_t* out_i,
                int32_t* out_j, double* out_v, double* out_mag);

/* MTTKRP A_ij = sum_kl B_ikl C_kj D_lj (Section 5.3), unfactored definition.
 * C: dim1 x J, D: dim2 x J row-major in the dtype of B; A, mag: dim0 x J. */
void orc_mttkrp(const orc_tensor* B, const void* C, const void* D, int32_t J,
                int64_t dim0, double* A, double* mag);

/* ---- plain per-format loop nests (what the paper's generated code does,
 * Section 5.2 / 5.3), native dtype, single thread. Timed as the CPU baseline
 * and cross-checked against the definitions above. ---- */
/* Threads used by the loops above that are parallel over disjoint outputs: effective only in
 * the build with -fopenmp (n <= 0 leaves the setting alone); returns the number in effect. */
int32_t orc_set_threads(int32_t n);
void orc_plain_spmv_csr(int64_t N, const int32_t* pos, const int32_t* crd,
                        const void* vals, const void* x, void* y, int32_t is_f64);
void orc_plain_spmv_coo(int64_t N, int64_t nnz, const int32_t* row,
                        const int32_t* col, const void* vals, const void* x,
                        void* y, int32_t is_f64);
void orc_plain_spmv_dia(int64_t N, int64_t M, int64_t K, const int32_t* offset,
                        const void* vals, const void* x, void* y, int32_t is_f64);
void orc_plain_spmv_ell(int64_t N, int64_t W, const int32_t* crd,
                        const void* vals, const void* x, void* y, int32_t is_f64);
int64_t orc_plain_ttv_coo(int64_t nnz, const int32_t* ci, const int32_t* cj,
                          const int32_t* ck, const void* vals, const void* c,
                          int32_t* out_i, int32_t* out_j, void* out_v,
                          int32_t is_f64);
void orc_plain_ttv_csf(int64_t nfib, const int32_t* pos2, const int32_t* crd2,
                       const void* vals, const void* c, void* out_v,
                       int32_t is_f64);
void orc_plain_mttkrp_coo(int64_t nnz, int64_t dim0, const int32_t* ci,
                          const int32_t* ck, const int32_t* cl, const void* vals,
                          const void* C, const void* D, int32_t J, void* A,
                          int32_t is_f64);
void orc_plain_spdm_coo(int64_t nnz, int64_t rows, const int32_t* row, const int32_t* col,
                        const void* vals, const void* C, int32_t J, void* A, int32_t is_f64);
void orc_plain_mttkrp_csf(int64_t dim0, const int32_t* pos0, const int32_t* crd0,
                          const int32_t* pos1, const int32_t* crd1,
                          const int32_t* pos2, const int32_t* crd2,
                          const void* vals, const void* C, const void* D,
                          int32_t J, void* A, int32_t is_f64);
#endif
