"""GPU parity: spt_mul (sparse A = B .* C, the intersection merge, on COO matrices, CSR matrices,
the CSR x COO pair of the paper's running example, and 3rd-order COO) and spt_add on operands
of mixed matrix formats, vs the oracle's two-way merge. Coordinates and pos bit-exact, values
within tolerance (each is one rounded product or sum, so results are in fact equal)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_add

pytestmark = pytest.mark.gpu


def _spec(fmt, N, M, r, c, v):
    return wl.csr_from_sorted_coo(N, M, r, c, v) if fmt == "csr" else wl.coo_spec(N, M, r, c, v)


def _overlapping(N, M, nb, nc, seed, dtype, share=0.5):
    """Two sorted matrices; about `share` of the smaller one's coordinates are also in the other."""
    r1, c1, v1 = wl.random_coo_entries(N, M, nb, seed=seed, dtype=dtype)
    r2, c2, v2 = wl.random_coo_entries(N, M, nc, seed=seed + 1, dtype=dtype)
    rng = np.random.default_rng(seed + 2)
    take = rng.random(len(v1)) < share * min(1.0, nc / max(nb, 1))
    key = np.concatenate([r2.astype(np.int64) * M + c2, r1[take].astype(np.int64) * M + c1[take]])
    vals = np.concatenate([v2, rng.uniform(-1, 1, int(take.sum())).astype(dtype)])
    key, first = np.unique(key, return_index=True)
    return (r1, c1, v1), ((key // M).astype(np.int32), (key % M).astype(np.int32), vals[first])


def _check(op, b, c, fmt, dtype, what, misalign=False):
    (ri, ci), rv, rm = (oracle.add if op == "add" else oracle.mul)(b, c)
    idx, gv = gpu_add(b, c, fmt, misalign=misalign, op=op)
    if fmt == "csr":
        pos = np.concatenate([[0], np.cumsum(np.bincount(ri, minlength=b.dims[0]))])
        assert np.array_equal(idx[0], pos), f"{what}: pos"
        assert np.array_equal(idx[1], ci), f"{what}: cols"
    else:
        assert np.array_equal(idx[0], ri) and np.array_equal(idx[1], ci), f"{what}: coordinates"
    assert_close(gv, rv, rm, dtype, what)
    return len(ri)


@pytest.mark.parametrize("fb,fc", [("coo", "coo"), ("csr", "csr"), ("csr", "coo"), ("coo", "csr")])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nb,nc", [(1, 1), (50, 70), (895, 897), (1792, 1792), (1793, 3000),
                                   (30_000, 41_000), (60_000, 500)])
def test_mul_matrices(fb, fc, dtype, nb, nc):
    N, M = 300, 257
    e1, e2 = _overlapping(N, M, nb, nc, 2000 + nb, dtype)
    b, c = _spec(fb, N, M, *e1), _spec(fc, N, M, *e2)
    n = _check("mul", b, c, fb, dtype, f"mul {fb}x{fc} {nb}x{nc}")
    if nb >= 50:
        assert 0 < n < min(len(e1[2]), len(e2[2])) + 1


@pytest.mark.parametrize("fb,fc", [("csr", "coo"), ("coo", "csr")])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_add_mixed_matrix_formats(fb, fc, dtype):
    N, M = 300, 257
    e1, e2 = _overlapping(N, M, 30_000, 41_000, 2100, dtype)
    _check("add", _spec(fb, N, M, *e1), _spec(fc, N, M, *e2), fb, dtype, f"add {fb}+{fc}")
    e1, e2 = _overlapping(N, M, 70, 5_000, 2101, dtype)
    _check("add", _spec(fb, N, M, *e1), _spec(fc, N, M, *e2), fb, dtype, f"add {fb}+{fc} small")


@pytest.mark.parametrize("fb,fc", [("csr", "coo"), ("csr", "csr"), ("coo", "coo")])
def test_mul_skewed_rows_empty_rows_and_misaligned(fb, fc):
    # power-law rows with long empty stretches: rows far longer than a chunk, many empty rows
    c4 = wl.config4(N=20_000, nnz_target=300_000, max_row=30_000, with_sorted=True)
    rs, cs, vs = c4["sorted"]
    N = 20_000
    r2, c2, v2 = wl.random_coo_entries(N, N, 150_000, seed=5, dtype=np.float64)
    half = slice(0, len(vs), 2)                 # plus every second entry of B itself: many twins
    key = np.concatenate([r2.astype(np.int64) * N + c2, rs[half].astype(np.int64) * N + cs[half]])
    vals = np.concatenate([v2, vs[half] * 0.5])
    key, first = np.unique(key, return_index=True)
    r2, c2, v2 = (key // N).astype(np.int32), (key % N).astype(np.int32), vals[first]
    b, c = _spec(fb, N, N, rs, cs, vs), _spec(fc, N, N, r2, c2, v2)
    n = _check("mul", b, c, fb, np.float64, f"mul {fb}x{fc} skewed")
    assert n >= len(vs[half]) - 10
    _check("mul", b, c, fb, np.float64, f"mul {fb}x{fc} skewed misaligned", misalign=True)
    if fb == fc:
        _check("mul", c, b, fb, np.float64, f"mul {fb}x{fc} skewed swapped")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nb,nc", [(100, 90), (20_000, 30_000), (5_000, 450_000)])
def test_mul_third_order(dtype, nb, nc):
    dims = (64, 64, 128) if nc > 100_000 else (40, 30, 50)
    bi, bj, bk, bv = wl.random_coo3_entries(dims, nb, 2200 + nb, dtype=dtype, dist="u11", skew=1.3)
    ci, cj, ck, cv = wl.random_coo3_entries(dims, nc, 2201 + nb, dtype=dtype, dist="u11")
    b, c = wl.coo3_spec(dims, bi, bj, bk, bv), wl.coo3_spec(dims, ci, cj, ck, cv)
    (ri, rj, rk), rv, rm = oracle.mul(b, c)
    idx, gv = gpu_add(b, c, "coo3", op="mul")
    assert np.array_equal(idx[0], ri) and np.array_equal(idx[1], rj) and np.array_equal(idx[2], rk)
    assert_close(gv, rv, rm, dtype, "mul coo3")
    idx2, gv2 = gpu_add(c, b, "coo3", op="mul")                         # commutative, bit for bit
    assert all(np.array_equal(a, b_) for a, b_ in zip(idx, idx2)) and np.array_equal(gv, gv2)


def test_mul_special_operands():
    dims = (30, 20, 25)
    bi, bj, bk, bv = wl.random_coo3_entries(dims, 6000, 7, dtype=np.float64, dist="u11")
    b = wl.coo3_spec(dims, bi, bj, bk, bv)
    idx, v = gpu_add(b, b, "coo3", op="mul")                            # B .* B: squares on B's structure
    assert np.array_equal(idx[0], bi) and np.array_equal(idx[2], bk) and np.array_equal(v, bv * bv)
    z = bv.copy()
    z[::2] = 0.0
    idx, v = gpu_add(b, wl.coo3_spec(dims, bi, bj, bk, z), "coo3", op="mul")   # explicit zeros stay stored
    assert len(v) == len(bv) and np.array_equal(v, bv * z)
    e = np.zeros(0, np.int32)
    empty = wl.coo3_spec(dims, e, e, e, np.zeros(0, np.float64))
    for x, y in ((b, empty), (empty, b), (empty, empty)):
        idx, v = gpu_add(x, y, "coo3", op="mul")
        assert len(v) == 0 and len(idx[0]) == 0
    # disjoint supports that interleave: nothing in common
    k1 = np.unique((bi.astype(np.int64) * 20 + bj) * 25 + 2 * (bk // 2), return_index=True)[1]
    d1 = wl.coo3_spec(dims, bi[k1], bj[k1], (2 * (bk // 2))[k1], bv[k1])
    sel = (2 * (bk // 2) + 1 < 25)[k1]
    d2 = wl.coo3_spec(dims, bi[k1][sel], bj[k1][sel], (2 * (bk // 2) + 1)[k1][sel], bv[k1][sel])
    idx, v = gpu_add(d1, d2, "coo3", op="mul")
    assert len(v) == 0
    # CSR with empty leading / trailing rows; an empty CSR operand leaves pos all zero
    N = 50
    top = wl.csr_from_sorted_coo(N, N, np.array([0, 0, 3], np.int32), np.array([1, 7, 2], np.int32), np.full(3, 3.0))
    bot = wl.csr_from_sorted_coo(N, N, np.array([3, 49], np.int32), np.array([2, 49], np.int32), np.full(2, 5.0))
    (pos, cols), v = gpu_add(top, bot, "csr", op="mul")
    assert list(cols) == [2] and list(v) == [15.0]
    assert pos[3] == 0 and pos[4] == 1 and pos[50] == 1
    none = wl.csr_from_sorted_coo(N, N, np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0))
    (pos, cols), v = gpu_add(top, none, "csr", op="mul")
    assert len(v) == 0 and not pos.any()


def test_mul_full_size():
    """Configuration 4's matrix as CSR (50M entries) times a COO matrix holding every third entry
    of it with other values plus 10M entries of its own (the CSR x COO pair of the running
    example, at full size): coordinates against numpy's intersection of the linearised keys,
    values against the definition through searchsorted."""
    c4 = wl.config4(with_sorted=True)
    rs, cs, vs = c4["sorted"]
    N = c4["coo"].dims[0]
    b = wl.csr_from_sorted_coo(N, N, rs, cs, vs)
    rng = np.random.default_rng(wl.SEED_BASE + 66)
    r2, c2, v2 = wl.random_coo_entries(N, N, 10_000_000, seed=wl.SEED_BASE + 67, dtype=np.float64)
    third = slice(0, len(vs), 3)
    key = np.concatenate([r2.astype(np.int64) * N + c2, rs[third].astype(np.int64) * N + cs[third]])
    vals = np.concatenate([v2, rng.uniform(0.5, 1.5, len(vs[third]))])
    key, first = np.unique(key, return_index=True)
    vals = vals[first]
    c = wl.coo_spec(N, N, (key // N).astype(np.int32), (key % N).astype(np.int32), vals)
    (pos, cols), gv = gpu_add(b, c, "csr", op="mul")
    kb = rs.astype(np.int64) * N + cs
    want = np.intersect1d(kb, key, assume_unique=True)
    assert len(gv) == len(want) and len(want) >= len(vs[third])
    rows = np.repeat(np.arange(N, dtype=np.int64), np.diff(pos.astype(np.int64)))
    assert np.array_equal(rows * N + cols, want)
    prod = vs[np.searchsorted(kb, want)] * vals[np.searchsorted(key, want)]
    assert np.array_equal(gv, prod)
