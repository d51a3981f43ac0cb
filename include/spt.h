/*
 * spt.h - C ABI of libspt: sparse tensor algebra kernels executed directly on
 * tensors described as coordinate hierarchies, one level format per dimension
 * (paper Section 3.1: dense, compressed, singleton, range, offset, hashed).
 *
 * Target: one AMD MI355X (gfx950). Every data pointer in this interface is a
 * DEVICE pointer unless its comment says "host". The structs themselves
 * (spt_tensor, spt_level) live in HOST memory and are read only during the
 * call. `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *
 * Ownership: the caller owns every buffer. The library never allocates or
 * frees device memory and keeps no state between calls; scratch memory comes
 * from the caller-supplied workspace `ws`, whose required size is returned by
 * spt_workspace_bytes(). `ws` must be 256-byte aligned. Calls enqueue work on
 * `stream` and return without synchronising.
 *
 * Errors: every entry point returns an spt_status. Only host-checkable
 * conditions are diagnosed (null pointers, unknown level kinds, illegal
 * kind/property combinations per Table 1, level compositions that are not
 * recognised, sizes that overflow int32 positions, workspace too small).
 * Device-side content (monotone pos, in-range crd) is NOT validated by the
 * operations themselves; spt_validate() checks it on request.
 * spt_last_error() returns a thread-local human readable message for the
 * last failing call on this thread.
 */
#ifndef SPT_H
#define SPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPT_OK = 0,
  SPT_ERR_INVALID_ARG = 1,
  SPT_ERR_UNSUPPORTED = 2,
  SPT_ERR_WORKSPACE = 3,
  SPT_ERR_DEVICE = 4
} spt_status;

/* The six level formats of Section 3.1 / Table 2. */
typedef enum {
  SPT_DENSE = 0,      /* coordinates [0,N); child position p*N + i            */
  SPT_COMPRESSED = 1, /* children of p are crd[pos[p] .. pos[p+1])            */
  SPT_SINGLETON = 2,  /* one child per parent at the same position: crd[p]    */
  SPT_RANGE = 3,      /* coordinates [max(0,-offset[d]), min(N, M-offset[d])) */
  SPT_OFFSET = 4,     /* one child per parent: parent coordinate + offset[d]  */
  SPT_HASHED = 5      /* segment of width M (=W) of an open-addressed table   */
} spt_level_kind;

typedef enum { SPT_F32 = 0, SPT_F64 = 1 } spt_dtype;

/* Level properties that are configurable per level (Section 3.3, Table 1).
 * full / branchless / compact follow from the kind. */
enum { SPT_ORDERED = 1, SPT_UNIQUE = 2 };

/* Entry order of the CSR produced by spt_coo_to_csr (the paper does not
 * describe the conversion; both orders are total and deterministic):
 *   ROW_COL    rows ascending, columns ascending inside a row, equal
 *              (row,col) pairs keep their input order (sorted CSR, the
 *              paper's default: ordered column level, Figure 4 caption).
 *   ROW_STABLE rows ascending, input order kept inside a row.
 * Duplicates are kept, never summed. */
typedef enum { SPT_ORDER_ROW_COL = 0, SPT_ORDER_ROW_STABLE = 1 } spt_order;

typedef enum {
  SPT_OP_SPMV = 0,
  SPT_OP_COO_TO_CSR = 1,
  SPT_OP_TTV = 2,
  SPT_OP_MTTKRP = 3,
  SPT_OP_INNERPROD = 4,
  SPT_OP_TTM = 5,
  SPT_OP_TO_CSF = 6,
  SPT_OP_TO_ELL = 7,
  SPT_OP_DIA_OFFSETS = 8,
  SPT_OP_TO_COO = 9,
  SPT_OP_SPMV_SPARSE_X = 10, /* spt_spmv_sparse_x: query on A */
  SPT_OP_SPDM = 11           /* spt_spdm: query on B with J */
  /* spt_add / spt_mul size their workspace from BOTH operands: spt_add_workspace_bytes(B, C) */
} spt_op;

/*
 * One coordinate hierarchy level (Section 3.1).
 *   kind   spt_level_kind
 *   mode   tensor dimension this level encodes (0-based), or -1 for a level
 *          that encodes no tensor dimension (DIA's diagonal index, ELL's slot)
 *   flags  SPT_ORDERED | SPT_UNIQUE
 *   N      dense/range: N_k of Table 2 (extent used in p*N+i);
 *          compressed/singleton/offset/hashed: size of the tensor dimension
 *   M      range: M_k of Table 2 (extent of the child dimension, DIA: #cols);
 *          hashed: W_k (table width per parent);
 *          compressed: number of parent positions (1 for a root level, #rows
 *          for CSR's column level, #entries of the level above for CSF);
 *          else 0
 *   pos    compressed: M + 1 int32 entries; else NULL
 *   crd    compressed/singleton/hashed: int32 coordinates; else NULL.
 *          A negative singleton coordinate marks padding (ELL) and the
 *          position is skipped, as the hashed level skips -1.
 *   offset range/offset: int32 offsets indexed by the coordinate of the
 *          enclosing diagonal level (DIA passes the same array to both)
 *   max_children  optional hint for a compressed level: an upper bound on the
 *          number of children of any one parent (CSR: the longest row), 0 =
 *          unknown. Like the level properties of Section 3.3 it is a declared
 *          invariant that only selects between loops. CSR SpMV has two: one that
 *          streams the entries of 256 rows at a time through LDS and lets one lane
 *          add up each row (best for short rows), and one that deals the entries
 *          out evenly whatever their rows (best for strongly skewed row lengths).
 *          Without the hint the mean row length nvals / rows decides (<= 32: the
 *          streamed loop); from 2^25 stored entries on, a kernel first looks at the
 *          entry counts of the 256-row blocks and the entry-balanced loop runs if one
 *          block holds more than 1/1536 of all entries. A declared bound <= 32
 *          selects the streamed loop, a larger one the entry-balanced loop. A bound
 *          that the data violates costs time, not correctness.
 *   crd_stride  elements of crd between the coordinates of consecutive positions: 0 or 1 =
 *          contiguous (struct of arrays). A larger stride describes the array-of-structs
 *          variant of Section 5.2, where one interleaved array holds the coordinates of each
 *          component side by side, (i, j) (i, j) ..., and level m points at element m of it
 *          with stride = order. Such tensors are "any composition" (spt_spmv, spt_to_coo,
 *          spt_mul_dense, spt_add_to_dense); spt_spmv on an array-of-structs COO matrix
 *          splits the coordinates into the workspace first and then runs the COO kernels.
 */
typedef struct {
  int32_t kind;
  int32_t mode;
  int32_t flags;
  int32_t max_children;
  int64_t N;
  int64_t M;
  const int32_t* pos;
  const int32_t* crd;
  const int32_t* offset;
  int64_t crd_stride;
} spt_level;

/*
 * A tensor = `order` tensor dimensions stored as `nlevels` levels, outermost
 * first, plus one contiguous values array with one entry per leaf position.
 * Recognised compositions (D dense, C compressed, S singleton, R range,
 * O offset; ~U = not flagged unique):
 *   CSR   (D rows, C cols)                        vals[nnz]
 *   COO   (C~U rows with pos=[0,nnz], S cols)     vals[nnz]
 *   DIA   (D diagonals K, R rows, O cols)         vals[K*N], cell (d,i) at d*N+i
 *   ELL   (D slots W, D rows, S cols)             vals[W*N], cell (k,i) at k*N+i
 *   COO3  (C~U, S~U, S)                           vals[nnz]
 *   CSF3  (C, C, C)                               vals[nnz]
 *   CSC   (D cols, C rows), the levels in the order (mode 1, mode 0); vals[nnz] in column
 *         order. spt_spmv only (columns expanded from pos, then binned by row like an
 *         unordered COO), otherwise any composition
 *   DCSR  (C rows with pos=[0,stored rows], C cols) vals[nnz]; spt_spmv only (a fast path
 *         when the row level is flagged unique), otherwise any composition
 *   BCSR  (D block rows, C block cols, D b1, D b2) vals[nblocks*b1*b2], blocks row-major;
 *         a blocked matrix cast as a 4th-order tensor (Section 3.2): order = 4, modes
 *         0..3 = (block row, block column, row in block, column in block), and component
 *         (i1, j1, i2, j2) is matrix element (i1*b1 + i2, j1*b2 + j2). spt_spmv only.
 * spt_spmv and spt_to_coo also accept every other legal composition ("any composition"
 * below); the remaining operations return SPT_ERR_UNSUPPORTED for them.
 *
 * Any composition: level 0 is dense, compressed (M = 1) or hashed; a range level needs a level
 * above it and an offset level two (their coordinates are computed from those levels'
 * coordinates, Table 2); every tensor dimension is encoded by exactly one level; dense and
 * range levels have N > 0 and hashed levels M > 0 when values are stored. nvals is the number
 * of leaf positions (positions of the last level), whether or not each holds a component.
 */
typedef struct {
  int32_t order;   /* number of tensor dimensions (1..3; 4 for a blocked matrix) */
  int32_t nlevels; /* number of levels (2..4) */
  int32_t dtype;   /* spt_dtype of vals and of every dense operand */
  int32_t reserved;
  spt_level level[4];
  const void* vals;
  int64_t nvals; /* number of entries of vals */
} spt_tensor;

/*
 * y = A x (Section 5.2, SpMV on COO/CSR/DIA/ELL). x: dense, one entry per
 * column; y: dense, one entry per row, OVERWRITTEN (rows without entries get
 * 0). Every stored entry counts (duplicates add up). COO flagged SPT_ORDERED
 * on its row level runs a deterministic segmented reduction; without the flag
 * the entries are accumulated with floating-point atomics (any order).
 * DCSR (compressed rows flagged SPT_UNIQUE, compressed cols) runs the CSR kernels over the
 * stored rows and places each sum at its row coordinate (deterministic; workspace from
 * spt_workspace_bytes(SPT_OP_SPMV, ...)). CSC has its columns written out of pos into the
 * workspace and its entries binned by row like an unordered COO; an array-of-structs COO
 * matrix (crd_stride = 2 on both levels) has its pairs split into the workspace and then runs
 * as COO. Both need the workspace the query returns. Any other composition of levels that stores a
 * matrix (dense, hashed rows or columns, DCSR with repeated row coordinates, ...) is
 * evaluated by reading the level functions of Table 2 per stored value, again with
 * floating-point atomics; it needs no workspace.
 * A blocked matrix (order 4, Section 3.2): x has (block columns * b2) entries, y has
 * (block rows * b1). BCSR with block edges up to 64 has a kernel of its own
 * (deterministic, workspace from spt_workspace_bytes(SPT_OP_SPMV, ...)); BCSR with larger
 * blocks and every other 4-level composition of a blocked matrix (e.g. CSB = dense, dense,
 * compressed non-unique, singleton) are read per stored value like any other composition.
 */
spt_status spt_spmv(const spt_tensor* A, const void* x, void* y, void* ws,
                    size_t ws_bytes, void* stream);

/*
 * spt_spmv for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same operands, result and
 * errors as spt_spmv; the scratch memory comes from a fixed array of
 * SPT_STATIC_SCRATCH_BYTES in device memory that belongs to the library's code object (every
 * GPU the library runs on holds its own copy until the process ends). The call allocates
 * nothing and frees nothing. An operand whose spt_workspace_bytes(SPT_OP_SPMV, ...) exceeds
 * SPT_STATIC_SCRATCH_BYTES is refused with SPT_ERR_WORKSPACE (CSR, ordered COO, DIA, ELL of
 * any size fit; the binned scatter of a large unordered COO does not). The array's address
 * is looked up on the first call on each device, so make that first call outside a graph
 * capture. All calls on one GPU share the array: calls that overlap in time on one GPU
 * (different streams, or threads) race; calls on one stream are ordered and safe.
 */
#define SPT_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
spt_status spt_spmv_static(const spt_tensor* A, const void* x, void* y, void* stream);

/*
 * y = A x with A in CSR and x stored as a 1st-order tensor (Section 5.4, Figure
 * 16: dense array vs sparse vector vs hash map as the format of x):
 *   sparse vector  one compressed level, ordered and unique: pos = [0, nnz_x]
 *                  (M = 1 parent), crd ascending, vals[nnz_x]
 *   hash map       one hashed level of width W = level.M: crd[W] with -1 = empty
 *                  bucket, vals[W]; coordinate i lives at the first matching slot
 *                  at or after i % W, probing linearly with wrap (locate, Table 2)
 * x.nvals = number of entries of x's vals (nnz_x or W); same dtype as A.
 * Every stored entry of A locates its column in x; absent coordinates count as
 * 0. y is overwritten. Workspace: SPT_OP_SPMV_SPARSE_X on A.
 */
spt_status spt_spmv_sparse_x(const spt_tensor* A, const spt_tensor* x, void* y, void* ws,
                             size_t ws_bytes, void* stream);

/*
 * COO -> CSR (the conversion of Section 5.4 / Figure 14; pos holds what Table 3's
 * append_edges + append_finalize produce, the running sum of the per-row counts).
 * pos_out[N+1], crd_out[nnz], vals_out[nnz]. If both COO levels are flagged
 * SPT_ORDERED the sort is skipped. Index outputs are exact.
 */
spt_status spt_coo_to_csr(const spt_tensor* A_coo, int32_t order /*spt_order*/,
                          int32_t* pos_out, int32_t* crd_out, void* vals_out,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * TTV, A_ij = sum_k B_ijk c_k (Section 5.3), contracting the dimension of B's
 * last level with the dense vector c. B must be ordered.
 *  COO3 input: output is COO sorted by (i,j) with one entry per distinct (i,j)
 *    that has a stored entry: out_crd0/out_crd1/out_vals have capacity nnz,
 *    *out_nnz_dev (device int64) receives the number of entries.
 *  CSF3 input: the output shares B's two upper levels; out_vals has one entry
 *    per position of level 1 (= B.level[2].M entries); out_crd0/out_crd1 are
 *    ignored and may be NULL; *out_nnz_dev receives that count if non-NULL.
 */
spt_status spt_ttv(const spt_tensor* B, const void* c, int32_t* out_crd0,
                   int32_t* out_crd1, void* out_vals, int64_t* out_nnz_dev,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * MTTKRP, A_ij = sum_kl B_ikl C_kj D_lj (Section 5.3), output dimension = the
 * dimension of B's first level. C: (dim of level 1) x J, D: (dim of level 2)
 * x J, A_out: (dim of level 0) x J, all dense row-major, A_out OVERWRITTEN
 * (rows without entries get 0). B is COO3 or CSF3, ordered. 1 <= J <= 1024.
 */
spt_status spt_mttkrp(const spt_tensor* B, const void* C, const void* D,
                      int32_t J, void* A_out, void* ws, size_t ws_bytes,
                      void* stream);

/*
 * SpDM, A = B C (Section 5.2, Figure 11): B an ordered COO matrix (N x M), C dense
 * M x J, A_out dense N x J, both row-major; A_out is OVERWRITTEN (rows of B
 * without entries give zero rows). 1 <= J <= 1024. Workspace: SPT_OP_SPDM with J.
 */
spt_status spt_spdm(const spt_tensor* B, const void* C, int32_t J, void* A_out, void* ws,
                    size_t ws_bytes, void* stream);

/*
 * TTM, A_ijk = sum_l B_ijl C_kl (Section 5.3), contracting the dimension of B's last level
 * with the dense matrix C: K x L row-major, L = that dimension, 1 <= K <= 1024. B: COO3 or
 * CSF3, ordered. Every (i,j) fibre of B that holds a stored entry yields all K values, so the
 * output stores its last dimension as a dense level: fibre f owns out_vals[f*K .. f*K+K).
 *  COO3 input: fibres ascend in (i,j); out_crd0/out_crd1 (capacity nnz) receive their
 *    coordinates, out_vals needs capacity nnz*K, *out_nfib_dev (device int64, required)
 *    receives the number of fibres.
 *  CSF3 input: the output shares B's two upper levels: one fibre per position of level 1
 *    (B.level[2].M fibres); out_crd0/out_crd1 are ignored, out_nfib_dev may be NULL.
 * Workspace: SPT_OP_TTM with J = K.
 */
spt_status spt_ttm(const spt_tensor* B, const void* C, int32_t K, int32_t* out_crd0,
                   int32_t* out_crd1, void* out_vals, int64_t* out_nfib_dev, void* ws,
                   size_t ws_bytes, void* stream);

/*
 * INNERPROD, alpha = sum_ijk B_ijk C_ijk (Section 5.3): B and C both COO3 (or both COO
 * matrices: alpha = sum_ij B_ij C_ij) of equal dimensions and dtype, every level ordered
 * and each coordinate stored at most once per operand. Only coordinates stored in both
 * contribute (the intersection merge of Section 4.4). *alpha_out: one DEVICE scalar of the
 * operands' dtype, overwritten (0 if either operand is empty). Products and sums are
 * formed in double. Workspace: query with SPT_OP_INNERPROD on B.
 */
spt_status spt_innerprod(const spt_tensor* B, const spt_tensor* C, void* alpha_out, void* ws,
                         size_t ws_bytes, void* stream);

/*
 * Packing ordered COO into the other formats (Section 3.4: a tensor is assembled level by
 * level, by appends where coordinates arrive in order and by inserts otherwise). Index
 * outputs are exact, values are copied bit for bit. Coordinates are assumed unique.
 *
 * spt_coo3_to_csf: B = COO3, every level ordered. Output = the three compressed levels of
 *   CSF: pos0[2], crd0 (capacity nnz), pos1 (nnz+1), crd1 (nnz), pos2 (nnz+1), crd2 (nnz),
 *   vals_out (nnz). counts_dev[2] (device int64) receives the number of entries of level 0
 *   (slices) and level 1 (fibres); pos1 holds slices+1 and pos2 fibres+1 valid entries.
 *   Workspace: SPT_OP_TO_CSF.
 *
 * spt_to_ell: A = COO matrix with both levels ordered, or CSR. W slots per row: cell (k, i)
 *   at k*N + i of crd_out / vals_out (W*N entries each) receives the k-th entry of row i,
 *   unused cells column -1 and value 0. *longest_dev (device int32) receives the longest
 *   row; if it exceeds W the entries beyond slot W-1 were left out. Workspace: SPT_OP_TO_ELL
 *   (needed for COO only).
 *
 * spt_to_hashed_rows: A = COO matrix (any order, entries with W > 0 and rows non-empty of
 *   slots). Output = (dense rows, hashed columns of width W): crd_out / vals_out with N*W
 *   entries each; Table 3's hashed insert: crd is filled with -1, then every entry takes the
 *   first slot at or after col % W (wrapping, inside its row's segment) that is empty or already
 *   holds its column. When two columns of a row collide, which gets the earlier slot is not
 *   fixed (any result is a table in which locate finds every stored column). *dropped_dev
 *   (device int32) receives the number of entries whose row segment was full. No workspace.
 *
 * spt_coo_dia_offsets: A = COO matrix (any order). The distinct values of col - row,
 *   ascending, go to offsets_out (at most cap of them); *K_dev (device int64) receives their
 *   number. Workspace: SPT_OP_DIA_OFFSETS.
 * spt_coo_to_dia: vals_out[K*N], cell (d, i) at d*N + i = the entry of row i on diagonal
 *   offsets[d] (device array, ascending, K entries), zero where none is stored; entries on
 *   other diagonals are skipped. Needs no workspace.
 */
spt_status spt_coo3_to_csf(const spt_tensor* B, int32_t* pos0, int32_t* crd0, int32_t* pos1,
                           int32_t* crd1, int32_t* pos2, int32_t* crd2, void* vals_out,
                           int64_t* counts_dev, void* ws, size_t ws_bytes, void* stream);
spt_status spt_to_ell(const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                      int32_t* longest_dev, void* ws, size_t ws_bytes, void* stream);
spt_status spt_to_hashed_rows(const spt_tensor* A, int32_t W, int32_t* crd_out, void* vals_out,
                              int32_t* dropped_dev, void* stream);
spt_status spt_coo_dia_offsets(const spt_tensor* A, int32_t* offsets_out, int64_t cap,
                               int64_t* K_dev, void* ws, size_t ws_bytes, void* stream);
spt_status spt_coo_to_dia(const spt_tensor* A, int32_t K, const int32_t* offsets, void* vals_out,
                          void* stream);

/*
 * Any composition -> COO, in storage order (Section 3.1: every format is a coordinate
 * hierarchy; its components are the root-to-leaf paths). T: order 1..3, any composition; or a
 * blocked matrix of order 4 (BCSR, CSB, ...), written as the matrix it stores: out_crd0 /
 * out_crd1 receive i1*b1 + i2 and j1*b2 + j2, every cell of a stored dense block counts.
 * out_crd0 .. out_crd[order-1] and out_vals need capacity nvals; components whose position
 * holds none (padding, empty buckets, cells outside a range level) are left out;
 * *out_nnz_dev (device int64) receives the number written. Workspace: SPT_OP_TO_COO.
 */
spt_status spt_to_coo(const spt_tensor* T, int32_t* out_crd0, int32_t* out_crd1, int32_t* out_crd2,
                      void* out_vals, int64_t* out_nnz_dev, void* ws, size_t ws_bytes, void* stream);

/*
 * A = B + C with a sparse result: matrix addition on COO or CSR (Section 5.2) and 3rd-order
 * PLUS on COO (Section 5.3). B and C: two matrices, each COO or CSR (the formats may differ;
 * the result takes B's), or two COO3 tensors; same dimensions and dtype, every level ordered,
 * each coordinate stored at most once per operand. The result has one entry per coordinate
 * stored in B or C (the union merge of Section 4.4), ordered, holding b, c or the rounded sum
 * b + c; sums that cancel stay stored.
 * Outputs need capacity nnz(B) + nnz(C) entries; *out_nnz_dev (device int64, required)
 * receives the entry count.
 *   B COO matrix: out_crd0 (rows), out_crd1 (cols), out_vals; out_pos, out_crd2 ignored.
 *   B COO3:       out_crd0, out_crd1, out_crd2, out_vals; out_pos ignored.
 *   B CSR:        out_pos[N+1] (what Table 3's append_edges + append_finalize produce), out_crd1 (cols), out_vals;
 *                 out_crd0, out_crd2 ignored.
 * Workspace: spt_add_workspace_bytes(B, C), about 4 bytes per stored entry of both operands
 * (CSR operands: up to 12).
 *
 * spt_mul: A = B .* C, the element-wise product with a sparse result (the running example of
 * Sections 1 and 4: a CSR matrix times a COO matrix, element by element). Operands, outputs,
 * capacities and workspace exactly as spt_add (min(nnz(B), nnz(C)) entries of capacity are
 * enough); the result has one entry per coordinate stored in BOTH operands (the intersection
 * merge of Section 4.4), holding the rounded product b * c; products that are zero stay stored.
 */
spt_status spt_add(const spt_tensor* B, const spt_tensor* C, int32_t* out_pos, int32_t* out_crd0,
                   int32_t* out_crd1, int32_t* out_crd2, void* out_vals, int64_t* out_nnz_dev,
                   void* ws, size_t ws_bytes, void* stream);
spt_status spt_mul(const spt_tensor* B, const spt_tensor* C, int32_t* out_pos, int32_t* out_crd0,
                   int32_t* out_crd1, int32_t* out_crd2, void* out_vals, int64_t* out_nnz_dev,
                   void* ws, size_t ws_bytes, void* stream);
size_t spt_add_workspace_bytes(const spt_tensor* B, const spt_tensor* C);

/*
 * Element-wise operations with a dense operand or a dense result, on matrices in ANY legal
 * composition of level formats (read per stored value through the level functions).
 * spt_mul_dense: A = B .* D (the first element-wise product of Figure 1). D: dense N x M,
 *   row-major with leading dimension ld >= M, B's dtype. The result has B's structure, so only
 *   values are produced: out_vals[p] = B.vals[p] * D(i, j) for the component (i, j) stored at
 *   leaf position p, 0 at positions that hold no component (ELL padding, empty hash buckets,
 *   cells outside a range level). out_vals: B.nvals entries; may not alias B.vals.
 * spt_add_to_dense: A = B + C with a dense result (the CSR + COO example of Section 4.4,
 *   Figure 9). A: dense N x M, row-major with leading dimension ld, OVERWRITTEN (cells that
 *   neither operand stores get 0). A dense result supports insertion at a computed position
 *   (Table 3), so the operands are not merged: each is walked on its own and its components
 *   are added with floating-point atomics (a cell receives at most one term per operand when
 *   coordinates are unique, so the result does not depend on the order). B, C: equal
 *   dimensions and dtype, formats may differ.
 * Neither needs a workspace.
 */
spt_status spt_mul_dense(const spt_tensor* B, const void* D, int64_t ld, void* out_vals, void* stream);
spt_status spt_add_to_dense(const spt_tensor* B, const spt_tensor* C, void* A, int64_t ld, void* stream);

/*
 * Device-side check of the CONTENT of T's level arrays (Section 3.1), which every other entry
 * point takes on trust: pos of each compressed level starts at 0, never decreases and ends at
 * the number of positions of its level (so the declared M of the level below is right);
 * stored coordinates lie in [0, N) (-1 is allowed where it marks padding: singleton and
 * hashed levels); inside every segment of a compressed level flagged SPT_ORDERED the
 * coordinates ascend (strictly if also SPT_UNIQUE); a COO tensor flagged ordered on all levels
 * is in lexicographic order; every DIA offset leaves at least one cell inside the matrix.
 * T: any composition spt_spmv / spt_to_coo accept. err_dev: two DEVICE int32: [0] receives the
 * number of violations found, [1] the OR of their kinds (SPT_BAD_*). Enqueues a few small
 * kernels and returns without synchronising; needs no workspace. Host-checkable problems are
 * reported through the status as everywhere else.
 */
enum { SPT_BAD_POS = 1, SPT_BAD_POS_END = 2, SPT_BAD_CRD = 4, SPT_BAD_ORDER = 8, SPT_BAD_OFFSET = 16 };
spt_status spt_validate(const spt_tensor* T, int32_t* err_dev, void* stream);

/* Workspace size in bytes for `op` on tensor T (J only for MTTKRP and TTM).
 * Returns 0 for invalid descriptors (spt_last_error says why). Never fails for
 * a valid one; the result is always >= 256. */
size_t spt_workspace_bytes(int32_t op, const spt_tensor* T, int32_t J);

/* Thread-local message of the last error raised on this thread ("" if none). */
const char* spt_last_error(void);

/* Library version string, e.g. "spt 0.1 gfx950". */
const char* spt_version(void);

/*
 * Measurement aids (no counterpart in the paper): the two access patterns that
 * bound every kernel above, isolated, so that a benchmark can state the
 * machine's achievable ceilings next to the kernels' figures.
 *  spt_probe_read   streams `bytes` bytes of src (16-byte aligned, bytes a
 *                   multiple of 16) once, lane_bytes = 4, 8 or 16 per lane
 *                   load; nothing is written except when the data sums to a
 *                   magic value (sink: device, >= 4 bytes).
 *  spt_probe_gather out[p] = table[idx[p]] for p < n (idx: device int32 in
 *                   range, table/out: dtype elements): the random cache-line
 *                   gather of x / factor rows.
 */
spt_status spt_probe_read(const void* src, size_t bytes, int32_t lane_bytes, void* sink,
                          void* stream);
spt_status spt_probe_gather(const int32_t* idx, int64_t n, const void* table, int32_t dtype,
                            void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPT_H */
