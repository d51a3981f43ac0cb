"""Seeded synthetic inputs and plain format descriptions.

This module holds DATA LAYOUT ONLY: it draws random coordinates and values and
lays them out as the level arrays (pos / crd / offset / vals) of each storage
format. It contains none of the arithmetic of the kernels under test; both the
CPU oracle and the GPU library are fed from here, and neither is imported.

The generated tensors stand in for the paper's evaluation inputs (Table 4:
SuiteSparse matrices and FROSTT tensors, which are not available offline):
uniform-random matrices, few-dense-diagonal matrices (like Lin / synth1 /
atmosmodd with 7 diagonals), bounded-row-length mesh-like matrices for ELL,
power-law web-like matrices, and skewed NELL-like 3rd-order tensors.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

DENSE, COMPRESSED, SINGLETON, RANGE, OFFSET, HASHED = range(6)
KIND_NAMES = ["dense", "compressed", "singleton", "range", "offset", "hashed"]


@dataclass
class LevelSpec:
    """One coordinate-hierarchy level (Section 3.1): kind + arrays + sizes."""
    kind: int
    mode: int
    N: int
    M: int = 0
    pos: Optional[np.ndarray] = None
    crd: Optional[np.ndarray] = None
    offset: Optional[np.ndarray] = None
    ordered: bool = True
    unique: bool = True
    max_children: int = 0     # optional declared bound on children per parent (0 = unknown)
    crd_stride: int = 1       # elements between consecutive positions in crd (> 1: interleaved)


@dataclass
class TensorSpec:
    """A tensor stored as a list of levels plus one values array."""
    dims: Tuple[int, ...]
    levels: List[LevelSpec]
    vals: np.ndarray
    name: str = ""

    @property
    def order(self) -> int:
        return len(self.dims)

    @property
    def dtype(self):
        return self.vals.dtype


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


# ---------------------------------------------------------------------------
# format layouts
# ---------------------------------------------------------------------------

def coo_spec(N, M, row, col, vals, ordered=True, name="coo") -> TensorSpec:
    """COO = (compressed non-unique rows with pos=[0,nnz], singleton cols)."""
    nnz = len(vals)
    return TensorSpec((N, M), [
        LevelSpec(COMPRESSED, 0, N, M=1, pos=_i32([0, nnz]), crd=_i32(row),
                  ordered=ordered, unique=False),
        LevelSpec(SINGLETON, 1, M, crd=_i32(col), ordered=ordered),
    ], np.ascontiguousarray(vals), name)


def coo_aos_spec(dims, coords, vals, ordered=True, name="coo-aos") -> TensorSpec:
    """Array-of-structs COO (Section 5.2): one array holds the coordinates of each component
    contiguously, (i, j[, k]) (i, j[, k]) ...; level m reads it from element m with stride
    order. The level arrays below are views into that one array."""
    order = len(dims)
    inter = np.ascontiguousarray(np.stack([_i32(c) for c in coords], axis=1).reshape(-1))
    nnz = len(vals)
    levels = [LevelSpec(COMPRESSED, 0, dims[0], M=1, pos=_i32([0, nnz]), crd=inter[0:], ordered=ordered,
                        unique=False, crd_stride=order)]
    for m in range(1, order):
        levels.append(LevelSpec(SINGLETON, m, dims[m], crd=inter[m:], ordered=ordered,
                                unique=m == order - 1, crd_stride=order))
    return TensorSpec(tuple(dims), levels, np.ascontiguousarray(vals), name)


def csr_spec(N, M, pos, crd, vals, ordered=True, unique=True, name="csr",
             max_row=0) -> TensorSpec:
    """CSR = (dense rows, compressed cols). max_row: declared bound on the row length
    when the construction guarantees one (0 = unknown)."""
    return TensorSpec((N, M), [
        LevelSpec(DENSE, 0, N),
        LevelSpec(COMPRESSED, 1, M, M=N, pos=_i32(pos), crd=_i32(crd),
                  ordered=ordered, unique=unique, max_children=max_row),
    ], np.ascontiguousarray(vals), name)


def dia_spec(N, M, offsets, diag_vals, name="dia") -> TensorSpec:
    """DIA = (dense diagonals, range rows, offset cols); cell (d,i) at d*N+i,
    column i+offset[d]; both lower levels share the offset array."""
    off = _i32(offsets)
    K = len(off)
    vals = np.ascontiguousarray(diag_vals).reshape(K * N)
    return TensorSpec((N, M), [
        LevelSpec(DENSE, -1, K),
        LevelSpec(RANGE, 0, N, M=M, offset=off),
        LevelSpec(OFFSET, 1, M, offset=off),
    ], vals, name)


def ell_spec(N, M, crd_wn, vals_wn, name="ell") -> TensorSpec:
    """ELL = (dense slots, dense rows, singleton cols); cell (k,i) at k*N+i,
    padding marked by column -1."""
    W = crd_wn.shape[0] if crd_wn.ndim == 2 else len(crd_wn) // max(N, 1)
    return TensorSpec((N, M), [
        LevelSpec(DENSE, -1, W),
        LevelSpec(DENSE, 0, N),
        LevelSpec(SINGLETON, 1, M, crd=_i32(crd_wn).reshape(W * N), ordered=False),
    ], np.ascontiguousarray(vals_wn).reshape(W * N), name)


def coo3_spec(dims, ci, cj, ck, vals, ordered=True, name="coo3") -> TensorSpec:
    """3rd-order COO = (compressed ~U, singleton ~U, singleton)."""
    nnz = len(vals)
    return TensorSpec(tuple(dims), [
        LevelSpec(COMPRESSED, 0, dims[0], M=1, pos=_i32([0, nnz]), crd=_i32(ci),
                  ordered=ordered, unique=False),
        LevelSpec(SINGLETON, 1, dims[1], crd=_i32(cj), ordered=ordered, unique=False),
        LevelSpec(SINGLETON, 2, dims[2], crd=_i32(ck), ordered=ordered),
    ], np.ascontiguousarray(vals), name)


def csf3_spec(dims, pos0, crd0, pos1, crd1, pos2, crd2, vals, name="csf3") -> TensorSpec:
    """CSF = (compressed, compressed, compressed)."""
    return TensorSpec(tuple(dims), [
        LevelSpec(COMPRESSED, 0, dims[0], M=1, pos=_i32(pos0), crd=_i32(crd0)),
        LevelSpec(COMPRESSED, 1, dims[1], M=len(crd0), pos=_i32(pos1), crd=_i32(crd1)),
        LevelSpec(COMPRESSED, 2, dims[2], M=len(crd1), pos=_i32(pos2), crd=_i32(crd2)),
    ], np.ascontiguousarray(vals), name)


def sparse_vector_spec(M, crd, vals, name="spvec") -> TensorSpec:
    """Sparse vector = one compressed level with pos = [0, nnz], ordered and unique."""
    return TensorSpec((M,), [LevelSpec(COMPRESSED, 0, M, M=1, pos=_i32([0, len(vals)]),
                                       crd=_i32(crd))], np.ascontiguousarray(vals), name)


def hash_vector_spec(M, crd, vals, W, name="hashvec") -> TensorSpec:
    """Hash-map vector = one hashed level of width W: coordinate i is stored at the first
    free slot at or after i % W (wrapping), empty slots hold -1 (Table 2 / Table 3)."""
    vals = np.asarray(vals)
    table = np.full(W, -1, np.int32)
    tv = np.zeros(W, vals.dtype)
    for i, v in zip(np.asarray(crd).tolist(), vals.tolist()):
        p = i % W
        while table[p] != -1:
            p = (p + 1) % W
        table[p] = i
        tv[p] = v
    return TensorSpec((M,), [LevelSpec(HASHED, 0, M, M=W, crd=table, ordered=False)], tv, name)


# ---- compositions without a kernel of their own (evaluated through the level functions) ----

def dcsr_from_sorted_coo(N, M, row, col, vals, name="dcsr") -> TensorSpec:
    """DCSR = (compressed rows, compressed cols): only rows that hold entries are stored."""
    row = np.asarray(row)
    rows, first = np.unique(row, return_index=True)
    pos1 = np.concatenate([first, [len(row)]]) if len(row) else np.zeros(1, np.int64)
    return TensorSpec((N, M), [
        LevelSpec(COMPRESSED, 0, N, M=1, pos=_i32([0, len(rows)]), crd=_i32(rows)),
        LevelSpec(COMPRESSED, 1, M, M=len(rows), pos=_i32(pos1), crd=_i32(col)),
    ], np.ascontiguousarray(vals), name)


def csc_from_coo(N, M, row, col, vals, name="csc") -> TensorSpec:
    """CSC = (dense cols, compressed rows): the levels store the dimensions in the order
    (1, 0); entries are laid out column-major."""
    row, col, vals = np.asarray(row), np.asarray(col), np.asarray(vals)
    order = np.lexsort((row, col))
    pos = np.searchsorted(col[order], np.arange(M + 1), side="left")
    return TensorSpec((N, M), [
        LevelSpec(DENSE, 1, M),
        LevelSpec(COMPRESSED, 0, N, M=M, pos=_i32(pos), crd=_i32(row[order])),
    ], np.ascontiguousarray(vals[order]), name)


def dense_matrix_spec(A, name="dense") -> TensorSpec:
    """(dense rows, dense cols): every cell is a leaf, row-major."""
    A = np.ascontiguousarray(A)
    N, M = A.shape
    return TensorSpec((N, M), [LevelSpec(DENSE, 0, N), LevelSpec(DENSE, 1, M)], A.reshape(-1), name)


def hashed_rows_from_coo(N, M, row, col, vals, W, name="dhash") -> TensorSpec:
    """(dense rows, hashed cols): every row owns a W-wide open-addressed table; column j sits
    at the first free slot at or after j % W of its row's segment (wrapping), -1 = empty."""
    vals = np.asarray(vals)
    table = np.full(N * W, -1, np.int32)
    tv = np.zeros(N * W, vals.dtype)
    for i, j, v in zip(np.asarray(row).tolist(), np.asarray(col).tolist(), vals.tolist()):
        q = j % W
        while table[i * W + q] != -1:
            q = (q + 1) % W
        table[i * W + q] = j
        tv[i * W + q] = v
    return TensorSpec((N, M), [
        LevelSpec(DENSE, 0, N),
        LevelSpec(HASHED, 1, M, M=W, crd=table, ordered=False),
    ], tv, name)


def sparse_dia_from_coo(N, M, row, col, vals, name="sdia") -> TensorSpec:
    """(dense diagonals, compressed rows, offset cols): DIA for sparsely filled diagonals; only
    the rows that hold an entry on a diagonal are stored, the column is row + offset[d]."""
    row, col, vals = np.asarray(row, np.int64), np.asarray(col, np.int64), np.asarray(vals)
    off = np.unique(col - row)
    d = np.searchsorted(off, col - row)
    order = np.lexsort((row, d))
    pos = np.searchsorted(d[order], np.arange(len(off) + 1), side="left")
    return TensorSpec((N, M), [
        LevelSpec(DENSE, -1, len(off)),
        LevelSpec(COMPRESSED, 0, N, M=len(off), pos=_i32(pos), crd=_i32(row[order])),
        LevelSpec(OFFSET, 1, M, offset=_i32(off)),
    ], np.ascontiguousarray(vals[order]), name)


def dcc3_from_sorted_coo(dims, ci, cj, ck, vals, name="dcc3") -> TensorSpec:
    """3rd-order (dense, compressed, compressed): CSF with a dense first level."""
    ci, cj = np.asarray(ci, np.int64), np.asarray(cj, np.int64)
    key = ci * dims[1] + cj
    fib, first = np.unique(key, return_index=True)
    pos2 = np.concatenate([first, [len(key)]]) if len(key) else np.zeros(1, np.int64)
    pos1 = np.searchsorted(fib // dims[1], np.arange(dims[0] + 1), side="left")
    return TensorSpec(tuple(dims), [
        LevelSpec(DENSE, 0, dims[0]),
        LevelSpec(COMPRESSED, 1, dims[1], M=dims[0], pos=_i32(pos1), crd=_i32(fib % dims[1])),
        LevelSpec(COMPRESSED, 2, dims[2], M=len(fib), pos=_i32(pos2), crd=_i32(ck)),
    ], np.ascontiguousarray(vals), name)


def bcsr_spec(Nb, Mb, b1, b2, pos, crd, blocks, name="bcsr") -> TensorSpec:
    """BCSR cast as a 4th-order tensor (block row, block col, row in block, col in block) =
    (dense, compressed, dense, dense): one dense b1 x b2 block of values, row-major, per stored
    block coordinate (Section 3.2)."""
    return TensorSpec((Nb, Mb, b1, b2), [
        LevelSpec(DENSE, 0, Nb),
        LevelSpec(COMPRESSED, 1, Mb, M=Nb, pos=_i32(pos), crd=_i32(crd)),
        LevelSpec(DENSE, 2, b1),
        LevelSpec(DENSE, 3, b2),
    ], np.ascontiguousarray(blocks).reshape(-1), name)


def _block_keys(N, M, row, col, b1, b2):
    Nb, Mb = -(-N // b1), -(-M // b2)
    row, col = np.asarray(row, np.int64), np.asarray(col, np.int64)
    return Nb, Mb, (row // b1) * Mb + col // b2, row % b1, col % b2


def bcsr_from_coo(N, M, row, col, vals, b1, b2, name="bcsr") -> TensorSpec:
    """The matrix's entries (distinct coordinates, any order) laid out as BCSR: every b1 x b2
    block that holds an entry is stored whole, cells without an entry hold 0."""
    Nb, Mb, bkey, ii, jj = _block_keys(N, M, row, col, b1, b2)
    ub, inv = np.unique(bkey, return_inverse=True)
    blocks = np.zeros((len(ub), b1, b2), np.asarray(vals).dtype)
    blocks[inv, ii, jj] = vals
    pos = np.concatenate([[0], np.cumsum(np.bincount(ub // Mb, minlength=Nb))])
    return bcsr_spec(Nb, Mb, b1, b2, pos, ub % Mb, blocks, name)


def csb_from_coo(N, M, row, col, vals, b1, b2, name="csb") -> TensorSpec:
    """CSB cast as a 4th-order tensor = (dense block rows, dense block columns, compressed
    non-unique rows in the block, singleton columns in the block): a dense grid of sparse blocks,
    each stored as a COO list (Section 3.2)."""
    Nb, Mb, bkey, ii, jj = _block_keys(N, M, row, col, b1, b2)
    o = np.lexsort((jj, ii, bkey))
    pos = np.concatenate([[0], np.cumsum(np.bincount(bkey, minlength=Nb * Mb))])
    return TensorSpec((Nb, Mb, b1, b2), [
        LevelSpec(DENSE, 0, Nb),
        LevelSpec(DENSE, 1, Mb),
        LevelSpec(COMPRESSED, 2, b1, M=Nb * Mb, pos=_i32(pos), crd=_i32(ii[o]), unique=False),
        LevelSpec(SINGLETON, 3, b2, crd=_i32(jj[o])),
    ], np.ascontiguousarray(np.asarray(vals)[o]), name)


def random_bcsr(Nb, Mb, b1, b2, lo, hi, seed, dtype=np.float64, dist="u11", band=0, with_csr=False):
    """Blocked matrix with lo..hi stored blocks per block row (FEM-like: `band` > 0 draws the
    block columns within +-band of the diagonal, else uniformly), full dense blocks.
    Returns {"bcsr", "x", "nblocks"} and, with_csr, the same matrix as CSR ("csr")."""
    rng = np.random.default_rng(seed)
    L = rng.integers(lo, hi + 1, Nb)
    brow = np.repeat(np.arange(Nb, dtype=np.int64), L)
    if band:
        bcol = np.clip(brow + rng.integers(-band, band + 1, len(brow)), 0, Mb - 1)
    else:
        bcol = rng.integers(0, Mb, len(brow))
    key = np.unique(brow * Mb + bcol)
    brow, bcol = key // Mb, key % Mb
    nb = len(key)
    L = np.bincount(brow, minlength=Nb)
    pos = np.concatenate([[0], np.cumsum(L)])
    blocks = _values(rng, nb * b1 * b2, dtype, dist).reshape(nb, b1, b2)
    out = {"bcsr": bcsr_spec(Nb, Mb, b1, b2, pos, bcol, blocks), "nblocks": nb,
           "x": dense_vector(Mb * b2, seed + 1000, dtype, dist)}
    if with_csr:
        # row (ib, ii) of the CSR twin lists the blocks of block row ib in order, each giving
        # its b2 cells of in-block row ii: a transposition (block, ii) -> (ii, block) per block row
        first = np.repeat(pos[:-1], L)                       # first block of each block's block row
        k = np.arange(nb, dtype=np.int64) - first            # rank of the block inside its block row
        Lb = np.repeat(L, L)                                 # blocks in that block row
        base = first * b1 * b2                               # CSR entries before the block row
        dst = (base[:, None, None] + np.arange(b1)[None, :, None] * (Lb * b2)[:, None, None]
               + (k * b2)[:, None, None] + np.arange(b2)[None, None, :])
        cvals = np.empty(nb * b1 * b2, dtype)
        ccol = np.empty(nb * b1 * b2, np.int32)
        cvals[dst.reshape(-1)] = blocks.reshape(-1)
        ccol[dst.reshape(-1)] = (bcol[:, None, None] * b2 + np.arange(b2)[None, None, :]
                                 + np.zeros((1, b1, 1), np.int64)).reshape(-1)
        cpos = np.concatenate([[0], np.cumsum(np.repeat(L * b2, b1))])
        out["csr"] = csr_spec(Nb * b1, Mb * b2, cpos, ccol, cvals, max_row=int(L.max()) * b2)
    return out


def random_sparse_vector(M, nnz, seed, dtype=np.float64, dist="u11"):
    """(sorted distinct coordinates, values) of a random sparse vector."""
    rng = np.random.default_rng(seed)
    crd = np.sort(rng.choice(M, size=min(nnz, M), replace=False))
    return _i32(crd), _values(rng, len(crd), dtype, dist)


def csr_from_sorted_coo(N, M, row, col, vals, name="csr") -> TensorSpec:
    """Lay a row-sorted entry list out as CSR (segment bounds from a sorted search)."""
    pos = np.searchsorted(np.asarray(row), np.arange(N + 1), side="left")
    return csr_spec(N, M, pos, col, vals, name=name)


def csf3_from_sorted_coo(dims, ci, cj, ck, vals, name="csf3") -> TensorSpec:
    """Lay a lexicographically sorted, duplicate-free entry list out as CSF."""
    ci, cj, ck = (np.asarray(a, dtype=np.int64) for a in (ci, cj, ck))
    nnz = len(ci)
    if nnz == 0:
        z = np.zeros(0, np.int32)
        return csf3_spec(dims, [0, 0], z, [0], z, [0], z, np.asarray(vals), name)
    new_i = np.ones(nnz, bool)
    new_i[1:] = ci[1:] != ci[:-1]
    new_ij = new_i.copy()
    new_ij[1:] |= cj[1:] != cj[:-1]
    fib_start = np.flatnonzero(new_ij)            # first entry of every (i,j) fiber
    slice_start_in_fibs = np.flatnonzero(new_i[fib_start])  # first fiber of every i
    crd0 = ci[fib_start][slice_start_in_fibs]
    pos0 = [0, len(crd0)]
    pos1 = np.append(slice_start_in_fibs, len(fib_start))
    crd1 = cj[fib_start]
    pos2 = np.append(fib_start, nnz)
    return csf3_spec(dims, pos0, crd0, pos1, crd1, pos2, ck, vals, name)


def csf3_with_empty_segments(dims, ci, cj, ck, vals, seed, extra_fibers, extra_slices,
                             name="csf3-gaps") -> TensorSpec:
    """CSF of a sorted, duplicate-free entry list whose compressed levels also hold EMPTY
    segments (Table 2: pos[p] = pos[p+1] is legal): `extra_fibers` (i,j) fibres without
    entries and `extra_slices` slices without fibres are mixed in at random coordinates, so
    empty fibres occur at the start, in the middle and at the end of slices, and whole slices
    consist of empty fibres only. The stored components are exactly the given entries."""
    rng = np.random.default_rng(seed)
    ci, cj, ck = (np.asarray(a, dtype=np.int64) for a in (ci, cj, ck))
    I, J = int(dims[0]), int(dims[1])
    real = np.unique(ci * J + cj)                       # fibres that hold entries
    gi = rng.integers(0, I, extra_fibers)
    if len(ci):                                         # most ghosts fall into slices that exist
        pick = rng.random(extra_fibers) < 0.8
        gi[pick] = ci[rng.integers(0, len(ci), int(pick.sum()))]
    ghosts = gi * J + rng.integers(0, J, extra_fibers)
    fibers = np.union1d(real, ghosts)                   # ascending (i,j), unique
    count = np.zeros(len(fibers), np.int64)
    if len(ci):
        np.add.at(count, np.searchsorted(fibers, ci * J + cj), 1)
    pos2 = np.concatenate(([0], np.cumsum(count)))
    fi = fibers // J
    slices = np.union1d(np.unique(fi), rng.integers(0, I, extra_slices))
    pos1 = np.searchsorted(fi, np.append(slices, I), side="left")
    return csf3_spec(dims, [0, len(slices)], slices, pos1, fibers % J, pos2, ck, vals, name)


# ---------------------------------------------------------------------------
# generic small random inputs (parity sweeps)
# ---------------------------------------------------------------------------

def _values(rng, n, dtype, dist):
    if dist == "u11":
        v = rng.uniform(-1.0, 1.0, n)
    elif dist == "u01":
        v = rng.uniform(0.0, 1.0, n)
    elif dist == "n01":
        v = rng.standard_normal(n)
    elif dist == "int":   # small integers: every partial sum is exact in fp32/fp64
        v = rng.integers(-4, 5, n).astype(np.float64)
    else:
        raise ValueError(dist)
    return v.astype(dtype)


def random_coo_entries(N, M, nnz, seed, dtype=np.float64, dist="u11",
                       duplicates=False, sort=True):
    """(row, col, vals) at uniform-random positions; distinct unless duplicates."""
    rng = np.random.default_rng(seed)
    if duplicates or N * M == 0:
        row = rng.integers(0, max(N, 1), nnz)
        col = rng.integers(0, max(M, 1), nnz)
    else:
        nnz = min(nnz, N * M)
        if N * M <= 4 * nnz + 64:
            key = rng.permutation(N * M)[:nnz]
        else:
            key = np.unique(rng.integers(0, N * M, int(nnz * 1.2) + 16))
            while len(key) < nnz:
                key = np.unique(np.concatenate([key, rng.integers(0, N * M, nnz)]))
            key = rng.permutation(key)[:nnz]
        row, col = key // M, key % M
    if sort:
        o = np.lexsort((col, row))
        row, col = row[o], col[o]
    vals = _values(rng, len(row), dtype, dist)
    return _i32(row), _i32(col), vals


def dense_vector(n, seed, dtype=np.float64, dist="u11"):
    return _values(np.random.default_rng(seed), n, dtype, dist)


def random_coo3_entries(dims, nnz, seed, dtype=np.float32, dist="u01", skew=None,
                        duplicates=False):
    """Sorted 3rd-order entries; mode 0 optionally Zipf(skew)-distributed."""
    rng = np.random.default_rng(seed)
    I, J, K = dims
    if skew:
        w = (np.arange(I) + 1.0) ** (-skew)
        cdf = np.cumsum(w / w.sum())
        ci = np.minimum(np.searchsorted(cdf, rng.random(nnz)), I - 1)
    else:
        ci = rng.integers(0, I, nnz)
    cj = rng.integers(0, J, nnz)
    ck = rng.integers(0, K, nnz)
    key = (ci.astype(np.int64) * J + cj) * K + ck
    key = np.sort(key) if duplicates else np.unique(key)
    ck = key % K
    cj = (key // K) % J
    ci = key // (K * J)
    vals = _values(rng, len(key), dtype, dist)
    return _i32(ci), _i32(cj), _i32(ck), vals


# ---------------------------------------------------------------------------
# the five benchmark configurations (full size by default, scalable)
# ---------------------------------------------------------------------------

SEED_BASE = 180410112


def config1(N=4096, nnz=40960, seed=SEED_BASE + 1):
    """Uniform-random fp64 matrix, distinct positions; COO sorted (row,col) + CSR."""
    row, col, vals = random_coo_entries(N, N, nnz, seed, np.float64, "u11")
    x = dense_vector(N, seed + 1000, np.float64, "u11")
    return {"coo": coo_spec(N, N, row, col, vals, name="c1-coo"),
            "csr": csr_from_sorted_coo(N, N, row, col, vals, name="c1-csr"),
            "x": x, "entries": (row, col, vals)}


def config2_offsets(N):
    """Offsets {0, +-1, +-~sqrt(N), +-N/2}: (0,1,1414,1000000) at N = 2e6."""
    a = max(2, int(np.floor(np.sqrt(N))))
    b = max(a + 1, N // 2)
    return np.array([-b, -a, -1, 0, 1, a, b], dtype=np.int64)


def config2(N=2_000_000, seed=SEED_BASE + 2, poison=False, dtype=np.float64):
    """Banded matrix with 7 densely filled diagonals, as DIA and as CSR."""
    rng = np.random.default_rng(seed)
    off = config2_offsets(N)
    K = len(off)
    i = np.arange(N, dtype=np.int64)
    diag = np.full((K, N), np.nan if poison else 0.0, dtype=dtype)
    valid = np.zeros((K, N), dtype=bool)
    for d in range(K):
        lo, hi = max(0, -off[d]), min(N, N - off[d])
        diag[d, lo:hi] = rng.uniform(-1.0, 1.0, hi - lo).astype(dtype)
        valid[d, lo:hi] = True
    # CSR of the same entries: row-major walk over (row, diagonal); offsets
    # ascend, so columns ascend inside a row.
    vt = valid.T
    cols = (i[:, None] + off[None, :])[vt]
    vals = np.ascontiguousarray(diag.T)[vt]
    pos = np.concatenate([[0], np.cumsum(vt.sum(axis=1))])
    x = dense_vector(N, seed + 1000, dtype, "u11")
    return {"dia": dia_spec(N, N, off, diag, name="c2-dia"),
            "csr": csr_spec(N, N, pos, cols, vals, name="c2-csr", max_row=K),
            "x": x, "nnz": int(pos[-1])}


def config3(N=1_000_000, lo=8, hi=32, seed=SEED_BASE + 3, dtype=np.float32):
    """Row lengths uniform in [lo,hi], distinct uniform columns sorted inside a
    row and left-packed; ELL (width = max length, pad col -1 / value 0) + CSR."""
    rng = np.random.default_rng(seed)
    M = N
    hi = min(hi, M)
    lo = min(lo, hi)
    L = rng.integers(lo, hi + 1, N)
    W = int(L.max()) if N else 0
    slot = np.arange(W)[None, :]
    live = slot < L[:, None]
    if M <= 64 * max(W, 1):              # small column range: draw without replacement
        cols = np.argsort(rng.random((N, M)), axis=1)[:, :W]
        cols[~live] = M                  # sentinel sorts to the end of the row
        cols.sort(axis=1)
    else:
        cols = rng.integers(0, M, (N, W))
        cols[~live] = M
        cols.sort(axis=1)
        while True:                      # redraw rows that hold a repeated column
            dup = (cols[:, 1:] == cols[:, :-1]) & live[:, 1:]
            bad = np.flatnonzero(dup.any(axis=1))
            if len(bad) == 0:
                break
            fresh = rng.integers(0, M, (len(bad), W))
            fresh[~live[bad]] = M
            fresh.sort(axis=1)
            cols[bad] = fresh
    v = rng.standard_normal((N, W)).astype(dtype)
    v[~live] = 0
    crd = np.where(live, cols, -1)
    x = dense_vector(M, seed + 1000, dtype, "n01")
    pos = np.concatenate([[0], np.cumsum(L)])
    return {"ell": ell_spec(N, M, np.ascontiguousarray(crd.T), np.ascontiguousarray(v.T),
                            name="c3-ell"),
            "csr": csr_spec(N, M, pos, crd[live], v[live], name="c3-csr", max_row=W),
            "x": x, "nnz": int(pos[-1]), "W": W}


def config4(N=4_000_000, nnz_target=60_000_000, max_row=200_000, zipf=1.8,
            seed=SEED_BASE + 4, dtype=np.float64, with_sorted=False):
    """Power-law row lengths (truncated Zipf, thinned to ~nnz_target entries),
    uniform distinct columns, entries shuffled: unsorted COO."""
    rng = np.random.default_rng(seed)
    M = N
    max_row = min(max_row, M)
    k = np.arange(1, max_row + 1, dtype=np.float64)
    w = k ** (-zipf)
    cdf = np.cumsum(w / w.sum())
    L = np.minimum(np.searchsorted(cdf, rng.random(N)), max_row - 1) + 1
    keep = min(1.0, nnz_target / float(L.sum()))
    L = rng.binomial(L, keep)
    row = np.repeat(np.arange(N, dtype=np.int64), L)
    col = rng.integers(0, M, len(row))
    key = np.unique(row * M + col)        # distinct columns inside every row (sorted)
    del row, col
    perm = rng.permutation(len(key))      # unsorted COO: entry p is sorted entry perm[p]
    row, col = _i32(key[perm] // M), _i32(key[perm] % M)
    vals = _values(rng, len(row), dtype, "u11")
    x = dense_vector(M, seed + 1000, dtype, "u11")
    out = {"coo": coo_spec(N, M, row, col, vals, ordered=False, name="c4-coo"),
           "x": x, "nnz": len(row), "max_row_len": int(L.max())}
    if with_sorted:                       # the same entries in (row, col) order
        vs = np.empty_like(vals)
        vs[perm] = vals
        out["sorted"] = (_i32(key // M), _i32(key % M), vs)
    return out


def config5(dims=(100_000, 80_000, 50_000), nnz=50_000_000, zipf=1.5, rank=32,
            seed=SEED_BASE + 5, dtype=np.float32):
    """Skewed 3rd-order tensor (mode 0 Zipf), as sorted COO and as CSF, plus the
    dense TTV vector and the two rank-`rank` factor matrices."""
    ci, cj, ck, vals = random_coo3_entries(dims, nnz, seed, dtype, "u01", skew=zipf)
    rng = np.random.default_rng(seed + 1000)
    c = rng.uniform(0, 1, dims[2]).astype(dtype)
    C = rng.uniform(0, 1, (dims[1], rank)).astype(dtype)
    D = rng.uniform(0, 1, (dims[2], rank)).astype(dtype)
    return {"coo": coo3_spec(dims, ci, cj, ck, vals, name="c5-coo"),
            "csf": csf3_from_sorted_coo(dims, ci, cj, ck, vals, name="c5-csf"),
            "c": c, "C": C, "D": D, "nnz": len(vals)}
