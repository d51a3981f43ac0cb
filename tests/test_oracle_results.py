"""Pins for the oracle's results: library routines (scipy.sparse, numpy dense
algebra), closed forms, exact-integer cases and cross-format agreement.
Each pin is chosen so that a dropped term, wrong sign/index or transposed
operand in oracle.c fails it. CPU only."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import workloads as wl


def _dense(N, M, r, c, v):
    D = np.zeros((N, M), np.float64)
    np.add.at(D, (r, c), v.astype(np.float64))
    return D


# ------------------------------------------------------------------ SpMV

@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("dup", [False, True])
def test_spmv_coo_csr_vs_dense_and_scipy(dtype, dup):
    N, M = 37, 53                                  # non-square: catches transposition
    r, c, v = wl.random_coo_entries(N, M, 400, seed=11, dtype=dtype, duplicates=dup)
    x = wl.dense_vector(M, 12, dtype)
    want = _dense(N, M, r, c, v) @ x.astype(np.float64)
    want_sp = sp.coo_matrix((v.astype(np.float64), (r, c)), shape=(N, M)).tocsr() @ x.astype(np.float64)
    for spec in (wl.coo_spec(N, M, r, c, v), wl.csr_from_sorted_coo(N, M, r, c, v)):
        y, mag = oracle.spmv(spec, x)
        np.testing.assert_allclose(y, want, rtol=0, atol=1e-13 * max(1.0, mag.max()))
        np.testing.assert_allclose(y, want_sp, rtol=0, atol=1e-13 * max(1.0, mag.max()))
        want_mag = _dense(N, M, r, c, np.abs(v)) @ np.abs(x.astype(np.float64))
        np.testing.assert_allclose(mag, want_mag, rtol=1e-12)


def test_spmv_unsorted_coo_is_order_independent():
    N, M = 20, 30
    r, c, v = wl.random_coo_entries(N, M, 150, seed=4)
    x = wl.dense_vector(M, 5)
    p = np.random.default_rng(0).permutation(len(v))
    y0, _ = oracle.spmv(wl.coo_spec(N, M, r, c, v), x)
    y1, _ = oracle.spmv(wl.coo_spec(N, M, r[p], c[p], v[p], ordered=False), x)
    np.testing.assert_allclose(y0, y1, rtol=0, atol=1e-15)


def test_spmv_closed_forms():
    N = 9
    eye = wl.coo_spec(N, N, np.arange(N), np.arange(N), np.ones(N))
    x = wl.dense_vector(N, 1)
    assert np.array_equal(oracle.spmv(eye, x)[0], x)                 # A = I  =>  y = x
    r, c, v = wl.random_coo_entries(7, 5, 20, seed=3)
    D = _dense(7, 5, r, c, v)
    spec = wl.csr_from_sorted_coo(7, 5, r, c, v)
    for j in range(5):                                               # x = e_j => column j
        e = np.zeros(5)
        e[j] = 1
        assert np.array_equal(oracle.spmv(spec, e)[0], D[:, j])
    np.testing.assert_allclose(oracle.spmv(spec, np.ones(5))[0], D.sum(1), atol=1e-15)
    y, _ = oracle.spmv(wl.csr_from_sorted_coo(4, 4, [], [], np.zeros(0)), np.ones(4))
    assert np.array_equal(y, np.zeros(4))                            # empty rows give 0


def test_spmv_exact_integer_case_is_bit_exact_in_every_format():
    c2 = wl.config2(N=64, seed=2)
    off = wl.config2_offsets(64)
    rng = np.random.default_rng(1)
    diag = c2["dia"].vals.reshape(len(off), 64).copy()
    diag[~np.isnan(diag)] = 0
    for d, o in enumerate(off):
        lo, hi = max(0, -o), min(64, 64 - o)
        diag[d, lo:hi] = rng.integers(-4, 5, hi - lo)
    x = rng.integers(-4, 5, 64).astype(np.float64)
    dia = wl.dia_spec(64, 64, off, diag)
    want = np.zeros(64)
    for d, o in enumerate(off):
        for i in range(max(0, -o), min(64, 64 - o)):
            want[i] += diag[d, i] * x[i + o]
    assert np.array_equal(oracle.spmv(dia, x)[0], want)
    assert np.array_equal(oracle.plain_spmv(dia, x, "dia"), want)


def test_spmv_dia_vs_scipy_dia_and_csr_twin():
    N = 300
    c2 = wl.config2(N=N, seed=8, poison=True)
    off = wl.config2_offsets(N)
    x = c2["x"]
    y_dia, mag = oracle.spmv(c2["dia"], x)
    y_csr, _ = oracle.spmv(c2["csr"], x)
    assert np.isfinite(y_dia).all()                       # poison cells never read
    np.testing.assert_allclose(y_dia, y_csr, rtol=0, atol=1e-15 * mag.max())
    # scipy's DIA indexes its data by COLUMN: data[d, i+off] = our cell (d,i)
    dv = np.nan_to_num(c2["dia"].vals.reshape(len(off), N))
    data = np.zeros((len(off), N))
    for d, o in enumerate(off):
        lo, hi = max(0, -o), min(N, N - o)
        data[d, lo + o:hi + o] = dv[d, lo:hi]
    want = sp.dia_matrix((data, off), shape=(N, N)) @ x
    np.testing.assert_allclose(y_dia, want, rtol=0, atol=1e-14 * mag.max())
    # a single diagonal is an element-wise product with a shifted x
    one = wl.dia_spec(6, 9, [2], np.arange(1.0, 7.0)[None, :])
    xx = np.arange(10.0, 19.0)
    assert np.array_equal(oracle.spmv(one, xx)[0], np.arange(1.0, 7.0) * xx[2:8])


def test_spmv_dia_rectangular_and_out_of_range_diagonals():
    N, M = 5, 8
    off = np.array([-7, -1, 0, 3, 7, 12])                 # -7 and 12 lie fully outside
    diag = np.random.default_rng(3).uniform(-1, 1, (len(off), N))
    x = wl.dense_vector(M, 2)
    D = np.zeros((N, M))
    for d, o in enumerate(off):
        for i in range(N):
            if 0 <= i + o < M:
                D[i, i + o] += diag[d, i]
    y, _ = oracle.spmv(wl.dia_spec(N, M, off, diag), x)
    np.testing.assert_allclose(y, D @ x, atol=1e-15)


def test_spmv_ell_vs_csr_twin_and_padding_is_ignored():
    c3 = wl.config3(N=200, lo=0, hi=9, seed=6, dtype=np.float32)
    x = c3["x"]
    ell = c3["ell"]
    y_csr, mag = oracle.spmv(c3["csr"], x)
    y_ell, _ = oracle.spmv(ell, x)
    np.testing.assert_allclose(y_ell, y_csr, rtol=0, atol=1e-15 * max(mag.max(), 1))
    lv = c3["csr"].levels[1]
    want = sp.csr_matrix((c3["csr"].vals.astype(np.float64), lv.crd, lv.pos), shape=(200, 200)) @ x.astype(np.float64)
    np.testing.assert_allclose(y_csr, want, rtol=0, atol=1e-13 * max(mag.max(), 1))
    v = ell.vals.copy()
    v[ell.levels[2].crd < 0] = np.nan                     # poison the padding values
    poisoned = wl.TensorSpec(ell.dims, ell.levels, v)
    assert np.array_equal(oracle.spmv(poisoned, x)[0], y_ell)
    assert np.array_equal(oracle.plain_spmv(poisoned, x, "ell").astype(np.float64),
                          oracle.plain_spmv(ell, x, "ell").astype(np.float64))


@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-13), (np.float32, 2e-6)])
def test_plain_spmv_loops_agree_with_definition(dtype, tol):
    c1 = wl.config1(N=128, nnz=900, seed=21)
    c2 = wl.config2(N=257, seed=22, dtype=dtype)
    c3 = wl.config3(N=130, lo=1, hi=12, seed=23, dtype=dtype)
    cases = [(c2["dia"], c2["x"], "dia"), (c2["csr"], c2["x"], "csr"),
             (c3["ell"], c3["x"], "ell"), (c3["csr"], c3["x"], "csr")]
    if dtype == np.float64:
        cases += [(c1["coo"], c1["x"], "coo"), (c1["csr"], c1["x"], "csr")]
    for spec, x, fmt in cases:
        y, mag = oracle.spmv(spec, x)
        got = oracle.plain_spmv(spec, x, fmt).astype(np.float64)
        assert np.all(np.abs(got - y) <= tol * np.maximum(mag, 1e-30) + 1e-300), fmt


# ------------------------------------------------------------------ blocked matrices as 4th-order tensors

@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-15), (np.float32, 1e-15)])
@pytest.mark.parametrize("b1,b2", [(2, 3), (4, 4), (3, 1), (1, 5)])
def test_spmv_bcsr_vs_scipy_bsr_and_csr_twin(dtype, tol, b1, b2):
    Nb, Mb = 37, 29
    w = wl.random_bcsr(Nb, Mb, b1, b2, 0, 7, seed=91, dtype=dtype, with_csr=True)
    b, x = w["bcsr"], w["x"]
    lv = b.levels[1]
    y, mag = oracle.spmv_blocked(b, x)
    S = sp.bsr_matrix((b.vals.astype(np.float64).reshape(-1, b1, b2), lv.crd, lv.pos),
                      shape=(Nb * b1, Mb * b2))
    np.testing.assert_allclose(y, S @ x.astype(np.float64), rtol=0, atol=1e-13 * max(mag.max(), 1))
    np.testing.assert_allclose(y, S.toarray() @ x.astype(np.float64), rtol=0, atol=1e-13 * max(mag.max(), 1))
    np.testing.assert_allclose(mag, abs(S) @ np.abs(x.astype(np.float64)), rtol=0, atol=1e-13 * max(mag.max(), 1))
    y2, _ = oracle.spmv(w["csr"], x)                       # the same matrix entry by entry
    np.testing.assert_allclose(y, y2, rtol=0, atol=tol * max(mag.max(), 1))
    # x = e_c picks matrix column c, block structure and all
    c = 2 * b2 + (b2 - 1)
    e = np.zeros(Mb * b2, dtype)
    e[c] = 1
    np.testing.assert_array_equal(oracle.spmv_blocked(b, e)[0], S.toarray()[:, c])


def test_spmv_blocked_formats_of_one_matrix_agree():
    # BCSR (padded with explicit zeros) and CSB (sparse blocks) of a matrix whose size is no
    # multiple of the block size, against scipy on the plain entries
    N, M, b1, b2 = 50, 41, 4, 3
    r, c, v = wl.random_coo_entries(N, M, 400, seed=92, dtype=np.float64)
    x = wl.dense_vector(-(-M // b2) * b2, 93)
    want = sp.coo_matrix((v, (r, c)), shape=(N, -(-M // b2) * b2)).tocsr() @ x
    for spec in (wl.bcsr_from_coo(N, M, r, c, v, b1, b2), wl.csb_from_coo(N, M, r, c, v, b1, b2)):
        y, mag = oracle.spmv_blocked(spec, x)
        assert len(y) == -(-N // b1) * b1
        np.testing.assert_allclose(y[:N], want, rtol=0, atol=1e-13 * max(mag.max(), 1))
        assert not y[N:].any()
    # CSB stores exactly the entries; BCSR stores whole blocks
    assert len(wl.csb_from_coo(N, M, r, c, v, b1, b2).vals) == len(v)
    coords, vals = oracle.to_coo(wl.csb_from_coo(N, M, r, c, v, b1, b2))
    rows, cols = coords[0] * b1 + coords[2], coords[1] * b2 + coords[3]
    o = np.lexsort((cols, rows))
    assert np.array_equal(rows[o], r) and np.array_equal(cols[o], c) and np.array_equal(vals[o], v)


# ------------------------------------------------------------------ COO -> CSR

@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("dup", [False, True])
def test_coo_to_csr_vs_numpy_and_scipy(order, dup):
    N, M = 23, 17
    r, c, v = wl.random_coo_entries(N, M, 300, seed=31, duplicates=dup, sort=False)
    pos, crd, vout, perm = oracle.coo_to_csr(N, r, c, v, order)
    # numpy's lexsort is a stable indirect sort: the expected permutation
    want_perm = np.lexsort((c, r)) if order == 0 else np.argsort(r, kind="stable")
    assert np.array_equal(perm, want_perm)
    assert np.array_equal(crd, c[want_perm]) and np.array_equal(vout, v[want_perm])
    want_pos = np.concatenate([[0], np.cumsum(np.bincount(r, minlength=N))])
    assert np.array_equal(pos, want_pos)
    assert pos[0] == 0 and pos[-1] == len(r) and np.all(np.diff(pos) >= 0)
    if not dup and order == 0:
        m = sp.coo_matrix((v, (r, c)), shape=(N, M)).tocsr()
        m.sort_indices()
        assert np.array_equal(pos, m.indptr) and np.array_equal(crd, m.indices)
        assert np.array_equal(vout, m.data)
    if order == 0:
        for a, b in zip(pos[:-1], pos[1:]):
            assert np.all(np.diff(crd[a:b]) >= 0)


def test_coo_to_csr_fixed_point_and_edge_cases():
    r, c, v = wl.random_coo_entries(12, 12, 50, seed=33)
    pos, crd, vout, _ = oracle.coo_to_csr(12, r, c, v, 0)
    rows_back = np.repeat(np.arange(12), np.diff(pos))
    pos2, crd2, v2, perm2 = oracle.coo_to_csr(12, rows_back, crd, vout, 0)
    assert np.array_equal(pos, pos2) and np.array_equal(crd, crd2) and np.array_equal(vout, v2)
    assert np.array_equal(perm2, np.arange(len(v)))
    pos, crd, vout, _ = oracle.coo_to_csr(5, [], [], np.zeros(0), 0)
    assert np.array_equal(pos, np.zeros(6, np.int32)) and len(crd) == 0
    pos, crd, vout, _ = oracle.coo_to_csr(5, [3], [2], np.array([1.5], np.float32), 1)
    assert list(pos) == [0, 0, 0, 0, 1, 1] and list(crd) == [2] and vout[0] == np.float32(1.5)


# ------------------------------------------------------------------ TTV

def _dense3(dims, ci, cj, ck, v):
    B = np.zeros(dims, np.float64)
    np.add.at(B, (ci, cj, ck), v.astype(np.float64))
    return B


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_ttv_vs_dense_einsum(dtype):
    dims = (5, 4, 6)
    ci, cj, ck, v = wl.random_coo3_entries(dims, 70, seed=41, dtype=dtype, skew=1.5)
    c = wl.dense_vector(6, 42, dtype, "u01")
    B = _dense3(dims, ci, cj, ck, v)
    want = np.einsum("ijk,k->ij", B, c.astype(np.float64))
    fib = np.unique(ci.astype(np.int64) * 4 + cj)
    for spec in (wl.coo3_spec(dims, ci, cj, ck, v), wl.csf3_from_sorted_coo(dims, ci, cj, ck, v)):
        oi, oj, ov, om = oracle.ttv(spec, c)
        assert len(oi) == len(fib)                                 # one entry per stored fiber
        assert np.array_equal(oi.astype(np.int64) * 4 + oj, fib)   # ascending (i,j)
        np.testing.assert_allclose(ov, want[oi, oj], rtol=0, atol=1e-14 * om.max())
    # plain loops
    coo = wl.coo3_spec(dims, ci, cj, ck, v)
    csf = wl.csf3_from_sorted_coo(dims, ci, cj, ck, v)
    pi, pj, pv = oracle.plain_ttv(coo, c, "coo")
    tol = 1e-13 if dtype == np.float64 else 2e-6
    assert np.array_equal(pi, oi) and np.array_equal(pj, oj)
    assert np.all(np.abs(pv - ov) <= tol * om)
    assert np.all(np.abs(oracle.plain_ttv(csf, c, "csf") - ov) <= tol * om)


def test_ttv_closed_forms():
    dims = (4, 3, 5)
    ci, cj, ck, v = wl.random_coo3_entries(dims, 30, seed=43, dtype=np.float64)
    B = _dense3(dims, ci, cj, ck, v)
    spec = wl.coo3_spec(dims, ci, cj, ck, v)
    oi, oj, ov, _ = oracle.ttv(spec, np.ones(5))
    np.testing.assert_allclose(ov, B.sum(2)[oi, oj], atol=1e-15)     # c = 1: fiber sums
    e = np.zeros(5)
    e[2] = 1
    oi, oj, ov, _ = oracle.ttv(spec, e)
    assert np.array_equal(ov, B[:, :, 2][oi, oj])                    # c = e_k: slice k
    # a fiber whose sum is 0 is still emitted (structure comes from coordinates)
    z = wl.coo3_spec((2, 2, 2), [0, 0], [1, 1], [0, 1], np.array([1.0, -1.0]))
    oi, oj, ov, _ = oracle.ttv(z, np.ones(2))
    assert list(oi) == [0] and list(oj) == [1] and ov[0] == 0.0
    assert len(oracle.ttv(wl.coo3_spec((2, 2, 2), [], [], [], np.zeros(0)), np.ones(2))[0]) == 0


# ------------------------------------------------------------------ MTTKRP

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("J", [1, 3, 8])
def test_mttkrp_vs_dense_einsum_and_khatri_rao(dtype, J):
    dims = (5, 4, 6)
    ci, ck, cl, v = wl.random_coo3_entries(dims, 80, seed=51, dtype=dtype, skew=1.5)
    rng = np.random.default_rng(52)
    Cm = rng.uniform(0, 1, (4, J)).astype(dtype)
    Dm = rng.uniform(0, 1, (6, J)).astype(dtype)
    B = _dense3(dims, ci, ck, cl, v)
    C64, D64 = Cm.astype(np.float64), Dm.astype(np.float64)
    want = np.einsum("ikl,kj,lj->ij", B, C64, D64)
    # matricised form: B_(0) (I x KL) times the Khatri-Rao product (KL x J)
    kr = (C64[:, None, :] * D64[None, :, :]).reshape(4 * 6, J)
    np.testing.assert_allclose(B.reshape(5, 24) @ kr, want, atol=1e-13)
    coo = wl.coo3_spec(dims, ci, ck, cl, v)
    csf = wl.csf3_from_sorted_coo(dims, ci, ck, cl, v)
    tol = 1e-13 if dtype == np.float64 else 4e-6
    for spec in (coo, csf):
        A, mag = oracle.mttkrp(spec, Cm, Dm)
        np.testing.assert_allclose(A, want, rtol=0, atol=1e-14 * mag.max())
    for spec, fmt in ((coo, "coo"), (csf, "csf")):
        P = oracle.plain_mttkrp(spec, Cm, Dm, fmt).astype(np.float64)
        assert np.all(np.abs(P - A) <= tol * np.maximum(mag, 1e-30) + 1e-300), fmt


def test_mttkrp_closed_forms():
    dims = (4, 3, 5)
    ci, ck, cl, v = wl.random_coo3_entries(dims, 30, seed=53, dtype=np.float64)
    B = _dense3(dims, ci, ck, cl, v)
    spec = wl.coo3_spec(dims, ci, ck, cl, v)
    A, _ = oracle.mttkrp(spec, np.ones((3, 1)), np.ones((5, 1)))
    np.testing.assert_allclose(A[:, 0], B.sum((1, 2)), atol=1e-15)    # slice sums
    # D = 1 reduces MTTKRP to (TTV with ones) followed by a matrix product
    Cm = np.random.default_rng(1).uniform(0, 1, (3, 2))
    A, _ = oracle.mttkrp(spec, Cm, np.ones((5, 2)))
    np.testing.assert_allclose(A, B.sum(2) @ Cm, atol=1e-14)
    # integer data: exact regardless of summation order
    vi = np.random.default_rng(2).integers(-3, 4, len(v)).astype(np.float64)
    Ci = np.random.default_rng(3).integers(-3, 4, (3, 4)).astype(np.float64)
    Di = np.random.default_rng(4).integers(-3, 4, (5, 4)).astype(np.float64)
    si = wl.coo3_spec(dims, ci, ck, cl, vi)
    want = np.einsum("ikl,kj,lj->ij", _dense3(dims, ci, ck, cl, vi), Ci, Di)
    assert np.array_equal(oracle.mttkrp(si, Ci, Di)[0], want)
    assert np.array_equal(oracle.plain_mttkrp(si, Ci, Di, "coo"), want)


def test_csf_with_empty_fibres_and_slices_vs_dense_einsum():
    """A compressed level may hold empty segments (Table 2: pos[p] = pos[p+1]): empty fibres at
    the start, middle and end of slices and slices without fibres change nothing."""
    dims = (40, 9, 7)
    ci, ck, cl, v = wl.random_coo3_entries(dims, 120, seed=61, dtype=np.float64, skew=1.5)
    gap = wl.csf3_with_empty_segments(dims, ci, ck, cl, v, seed=62, extra_fibers=150, extra_slices=12)
    p1, p2 = np.asarray(gap.levels[1].pos), np.asarray(gap.levels[2].pos)
    lead = p1[:-1][np.diff(p1) > 0]
    assert (np.diff(p2) == 0).sum() > 50 and (np.diff(p1) == 0).sum() > 0   # gaps are really there
    assert (np.diff(p2)[lead] == 0).sum() > 0                               # ... also as first fibre of a slice
    B = _dense3(dims, ci, ck, cl, v)
    rng = np.random.default_rng(63)
    Cm, Dm, c = rng.uniform(0, 1, (9, 3)), rng.uniform(0, 1, (7, 3)), rng.uniform(0, 1, 7)
    A, mag = oracle.mttkrp(gap, Cm, Dm)
    np.testing.assert_allclose(A, np.einsum("ikl,kj,lj->ij", B, Cm, Dm), rtol=0, atol=1e-14 * mag.max())
    assert np.all(np.abs(oracle.plain_mttkrp(gap, Cm, Dm, "csf") - A) <= 1e-13 * mag + 1e-300)
    oi, oj, ov, om = oracle.ttv(gap, c)
    want = np.einsum("ijk,k->ij", B, c)
    assert np.array_equal(oi.astype(np.int64) * 9 + oj, np.unique(ci.astype(np.int64) * 9 + ck))
    np.testing.assert_allclose(ov, want[oi, oj], rtol=0, atol=1e-14 * om.max())
    # the plain CSF loop writes one value per fibre position, 0 for the empty ones
    pv = oracle.plain_ttv(gap, c, "csf")
    fi = np.repeat(np.asarray(gap.levels[0].crd), np.diff(p1))
    np.testing.assert_allclose(pv, want[fi, np.asarray(gap.levels[1].crd)] * (np.diff(p2) > 0), atol=1e-14)
    Ck = rng.uniform(0, 1, (4, 7))
    ti, tj, tv, tm = oracle.ttm(gap, Ck)
    assert np.array_equal(ti, oi) and np.array_equal(tj, oj)
    np.testing.assert_allclose(tv, np.einsum("ijl,kl->ijk", B, Ck)[ti, tj], rtol=0, atol=1e-14 * tm.max())


# ------------------------------------------------------------------ SpMV with sparse / hashed x

@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_spmv_sparse_and_hashed_x_vs_dense_expansion(dtype):
    N, M = 41, 67
    r, c, v = wl.random_coo_entries(N, M, 500, seed=61, dtype=dtype)
    A = wl.csr_from_sorted_coo(N, M, r, c, v)
    xc, xv = wl.random_sparse_vector(M, 20, seed=62, dtype=dtype)
    xd = np.zeros(M, np.float64)
    xd[xc] = xv                                   # independent dense expansion of x
    want = _dense(N, M, r, c, v) @ xd
    for W in (20, 23, 64, 200):                   # full table, prime, power of two, sparse table
        y, mag = oracle.spmv_sparse_x(A, wl.hash_vector_spec(M, xc, xv, W))
        np.testing.assert_allclose(y, want, rtol=0, atol=1e-13 * max(mag.max(), 1))
    y, mag = oracle.spmv_sparse_x(A, wl.sparse_vector_spec(M, xc, xv))
    np.testing.assert_allclose(y, want, rtol=0, atol=1e-13 * max(mag.max(), 1))
    # agrees with the dense-x definition on the expanded vector, magnitudes included
    y2, mag2 = oracle.spmv(A, xd.astype(dtype))
    np.testing.assert_allclose(y, y2, rtol=0, atol=1e-13 * max(mag.max(), 1))
    np.testing.assert_allclose(mag, mag2, rtol=1e-12, atol=1e-300)
    # empty x gives y = 0
    y, _ = oracle.spmv_sparse_x(A, wl.sparse_vector_spec(M, [], np.zeros(0, dtype)))
    assert not y.any()
    y, _ = oracle.spmv_sparse_x(A, wl.hash_vector_spec(M, [], np.zeros(0, dtype), 7))
    assert not y.any()


# ------------------------------------------------------------------ SpDM

@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("J", [1, 5, 32])
def test_spdm_vs_scipy_and_dense(dtype, J):
    N, M = 29, 43
    r, c, v = wl.random_coo_entries(N, M, 300, seed=81, dtype=dtype, duplicates=True)
    Cm = np.random.default_rng(82).uniform(-1, 1, (M, J)).astype(dtype)
    C64 = Cm.astype(np.float64)
    want = _dense(N, M, r, c, v) @ C64
    want_sp = sp.coo_matrix((v.astype(np.float64), (r, c)), shape=(N, M)).tocsr() @ C64
    for spec in (wl.coo_spec(N, M, r, c, v), wl.csr_from_sorted_coo(N, M, r, c, v)):
        A, mag = oracle.spdm(spec, Cm)
        np.testing.assert_allclose(A, want, rtol=0, atol=1e-13 * max(mag.max(), 1))
        np.testing.assert_allclose(A, want_sp, rtol=0, atol=1e-13 * max(mag.max(), 1))
    tol = 1e-13 if dtype == np.float64 else 4e-6
    P = oracle.plain_spdm(wl.coo_spec(N, M, r, c, v), Cm).astype(np.float64)
    assert np.all(np.abs(P - A) <= tol * np.maximum(mag, 1e-30) + 1e-300)
    # J = 1 is SpMV; C = I reproduces the dense matrix
    y, _ = oracle.spmv(wl.coo_spec(N, M, r, c, v), Cm[:, 0].copy())
    np.testing.assert_allclose(A[:, 0], y, rtol=0, atol=1e-15 * max(mag.max(), 1))
    E, _ = oracle.spdm(wl.coo_spec(N, M, r, c, v), np.eye(M, dtype=dtype))
    assert np.array_equal(E, _dense(N, M, r, c, v))


# ------------------------------------------------------------------ INNERPROD

@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_innerprod_vs_dense(dtype):
    dims = (6, 5, 7)
    bi, bj, bk, bv = wl.random_coo3_entries(dims, 90, seed=91, dtype=dtype, skew=1.5)
    ci, cj, ck, cv = wl.random_coo3_entries(dims, 120, seed=92, dtype=dtype)
    B, Cd = _dense3(dims, bi, bj, bk, bv), _dense3(dims, ci, cj, ck, cv)
    want = float((B * Cd).sum())
    assert 0 < np.count_nonzero(B * Cd) < min(len(bv), len(cv))     # a proper partial overlap
    bcoo, ccoo = wl.coo3_spec(dims, bi, bj, bk, bv), wl.coo3_spec(dims, ci, cj, ck, cv)
    ccsf = wl.csf3_from_sorted_coo(dims, ci, cj, ck, cv)
    for c in (ccoo, ccsf):
        a, mag = oracle.innerprod(bcoo, c)
        assert abs(a - want) <= 1e-13 * max(mag, 1)
        assert abs(mag - float(np.abs(B * Cd).sum())) <= 1e-12 * max(mag, 1)
    assert oracle.innerprod(ccoo, bcoo)[0] == oracle.innerprod(bcoo, ccoo)[0]      # symmetric
    sq, _ = oracle.innerprod(bcoo, bcoo)                                           # <B,B> = sum v^2
    assert abs(sq - float((bv.astype(np.float64) ** 2).sum())) <= 1e-13 * sq
    e = np.zeros(0, int)
    assert oracle.innerprod(bcoo, wl.coo3_spec(dims, e, e, e, np.zeros(0, dtype)))[0] == 0.0
    # disjoint supports
    d1 = wl.coo3_spec((2, 2, 2), [0], [0], [0], np.ones(1, dtype))
    d2 = wl.coo3_spec((2, 2, 2), [1], [1], [1], np.ones(1, dtype))
    assert oracle.innerprod(d1, d2) == (0.0, 0.0)


# ------------------------------------------------------------------ TTM

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("K", [1, 3, 7])
def test_ttm_vs_dense_einsum(dtype, K):
    dims = (5, 4, 6)
    ci, cj, cl, v = wl.random_coo3_entries(dims, 70, seed=61, dtype=dtype, skew=1.5)
    Cm = np.random.default_rng(62 + K).uniform(-1, 1, (K, 6)).astype(dtype)     # C_kl: K x L, not square
    B = _dense3(dims, ci, cj, cl, v)
    want = np.einsum("ijl,kl->ijk", B, Cm.astype(np.float64))
    fib = np.unique(ci.astype(np.int64) * 4 + cj)
    for spec in (wl.coo3_spec(dims, ci, cj, cl, v), wl.csf3_from_sorted_coo(dims, ci, cj, cl, v)):
        oi, oj, ov, om = oracle.ttm(spec, Cm)
        assert np.array_equal(oi.astype(np.int64) * 4 + oj, fib)            # one fibre per stored (i,j), ascending
        assert ov.shape == (len(fib), K)
        np.testing.assert_allclose(ov, want[oi, oj, :], rtol=0, atol=1e-14 * max(om.max(), 1))
        magwant = np.einsum("ijl,kl->ijk", np.abs(B), np.abs(Cm.astype(np.float64)))
        np.testing.assert_allclose(om, magwant[oi, oj, :], rtol=1e-12)


def test_ttm_closed_forms():
    dims = (4, 3, 5)
    ci, cj, cl, v = wl.random_coo3_entries(dims, 30, seed=63, dtype=np.float64)
    B = _dense3(dims, ci, cj, cl, v)
    spec = wl.coo3_spec(dims, ci, cj, cl, v)
    oi, oj, ov, _ = oracle.ttm(spec, np.eye(5))                     # C = I: the fibres themselves
    assert np.array_equal(ov, B[oi, oj, :])
    c = wl.dense_vector(5, 64, np.float64, "u11")
    ti, tj, tv, _ = oracle.ttv(spec, c)                             # K = 1 is TTV with c = C[0,:]
    oi, oj, ov, _ = oracle.ttm(spec, c[None, :])
    assert np.array_equal(oi, ti) and np.array_equal(oj, tj) and np.array_equal(ov[:, 0], tv)
    sel = np.zeros((2, 5))
    sel[0, 3] = 1.0
    sel[1, 1] = 2.0
    oi, oj, ov, _ = oracle.ttm(spec, sel)                           # rows of C pick slices l = 3 and 2 * (l = 1)
    assert np.array_equal(ov[:, 0], B[oi, oj, 3]) and np.array_equal(ov[:, 1], 2 * B[oi, oj, 1])
    assert len(oracle.ttm(wl.coo3_spec((2, 2, 2), [], [], [], np.zeros(0)), np.ones((3, 2)))[0]) == 0


# ------------------------------------------------------------------ sparse add (union merge)

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_add_matrices_vs_scipy(dtype):
    N, M = 40, 53
    r1, c1, v1 = wl.random_coo_entries(N, M, 500, seed=71, dtype=dtype)
    r2, c2, v2 = wl.random_coo_entries(N, M, 700, seed=72, dtype=dtype)
    S = (sp.coo_matrix((v1.astype(np.float64), (r1, c1)), shape=(N, M)).tocsr() +
         sp.coo_matrix((v2.astype(np.float64), (r2, c2)), shape=(N, M)).tocsr())
    S.sort_indices()
    S = S.tocoo()                                    # row-major, columns ascending
    shared = len(r1) + len(r2) - S.nnz
    assert 0 < shared < min(len(r1), len(r2))        # a proper partial overlap
    bcoo, ccoo = wl.coo_spec(N, M, r1, c1, v1), wl.coo_spec(N, M, r2, c2, v2)
    bcsr, ccsr = wl.csr_from_sorted_coo(N, M, r1, c1, v1), wl.csr_from_sorted_coo(N, M, r2, c2, v2)
    for b, c in ((bcoo, ccoo), (bcsr, ccsr), (bcoo, ccsr)):
        (ri, ci), v, mag = oracle.add(b, c)
        assert np.array_equal(ri, S.row) and np.array_equal(ci, S.col)
        np.testing.assert_allclose(v, S.data, rtol=0, atol=1e-15)
    # magnitudes: |b| + |c|
    Sa = (abs(sp.coo_matrix((v1.astype(np.float64), (r1, c1)), shape=(N, M)).tocsr()) +
          abs(sp.coo_matrix((v2.astype(np.float64), (r2, c2)), shape=(N, M)).tocsr()))
    Sa.sort_indices()
    np.testing.assert_allclose(mag, Sa.tocoo().data, rtol=0, atol=1e-15)


def test_add_third_order_vs_dense_and_closed_forms():
    dims = (6, 5, 7)
    bi, bj, bk, bv = wl.random_coo3_entries(dims, 90, seed=73, dtype=np.float64, skew=1.5)
    ci, cj, ck, cv = wl.random_coo3_entries(dims, 120, seed=74, dtype=np.float64)
    b, c = wl.coo3_spec(dims, bi, bj, bk, bv), wl.coo3_spec(dims, ci, cj, ck, cv)
    D = _dense3(dims, bi, bj, bk, bv) + _dense3(dims, ci, cj, ck, cv)
    support = (_dense3(dims, bi, bj, bk, np.ones(len(bv))) + _dense3(dims, ci, cj, ck, np.ones(len(cv)))) > 0
    (oi, oj, ok), v, _ = oracle.add(b, c)
    lin = (oi.astype(np.int64) * 5 + oj) * 7 + ok
    assert np.all(np.diff(lin) > 0)                                   # ordered, unique
    assert np.array_equal(lin, np.flatnonzero(support.ravel()))       # exactly the union
    np.testing.assert_allclose(v, D[oi, oj, ok], rtol=0, atol=1e-15)
    # commutative in coordinates and values
    (pi, pj, pk), pv, _ = oracle.add(c, b)
    assert np.array_equal(pi, oi) and np.array_equal(pj, oj) and np.array_equal(pk, ok) and np.array_equal(pv, v)
    # B + B = 2B on B's structure; B + (-B) keeps the structure with explicit zeros
    (qi, qj, qk), qv, _ = oracle.add(b, b)
    assert np.array_equal(qi, bi) and np.array_equal(qk, bk) and np.array_equal(qv, 2 * bv)
    neg = wl.coo3_spec(dims, bi, bj, bk, -bv)
    (zi, _, _), zv, zm = oracle.add(b, neg)
    assert len(zi) == len(bv) and np.all(zv == 0) and np.array_equal(zm, 2 * np.abs(bv))
    # empty operand: the other one unchanged
    e = np.zeros(0, int)
    (ei, ej, ek), ev, _ = oracle.add(b, wl.coo3_spec(dims, e, e, e, np.zeros(0)))
    assert np.array_equal(ei, bi) and np.array_equal(ej, bj) and np.array_equal(ek, bk) and np.array_equal(ev, bv)
    # CSF operands walk to the same result
    (fi, fj, fk), fv, _ = oracle.add(wl.csf3_from_sorted_coo(dims, bi, bj, bk, bv), c)
    assert np.array_equal(fi, oi) and np.array_equal(fk, ok) and np.array_equal(fv, v)


# ------------------------------------------------------------------ sparse multiply (intersection merge)

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_mul_matrices_vs_scipy(dtype):
    N, M = 40, 53
    r1, c1, v1 = wl.random_coo_entries(N, M, 500, seed=75, dtype=dtype)
    r2, c2, v2 = wl.random_coo_entries(N, M, 700, seed=76, dtype=dtype)
    B = sp.coo_matrix((v1.astype(np.float64), (r1, c1)), shape=(N, M)).tocsr()
    Cm = sp.coo_matrix((v2.astype(np.float64), (r2, c2)), shape=(N, M)).tocsr()
    S = B.multiply(Cm).tocsr()
    S.sort_indices()
    S = S.tocoo()
    assert 0 < S.nnz < min(len(r1), len(r2))          # a proper partial overlap
    bcoo, ccoo = wl.coo_spec(N, M, r1, c1, v1), wl.coo_spec(N, M, r2, c2, v2)
    bcsr, ccsr = wl.csr_from_sorted_coo(N, M, r1, c1, v1), wl.csr_from_sorted_coo(N, M, r2, c2, v2)
    for b, c in ((bcoo, ccoo), (bcsr, ccsr), (bcsr, ccoo), (bcoo, ccsr)):   # CSR x COO: the running example
        (ri, ci), v, mag = oracle.mul(b, c)
        assert np.array_equal(ri, S.row) and np.array_equal(ci, S.col)
        np.testing.assert_allclose(v, S.data, rtol=0, atol=1e-15)
        np.testing.assert_allclose(mag, np.abs(S.data), rtol=0, atol=1e-15)


def test_mul_third_order_vs_dense_and_closed_forms():
    dims = (6, 5, 7)
    bi, bj, bk, bv = wl.random_coo3_entries(dims, 90, seed=77, dtype=np.float64, skew=1.5)
    ci, cj, ck, cv = wl.random_coo3_entries(dims, 120, seed=78, dtype=np.float64)
    b, c = wl.coo3_spec(dims, bi, bj, bk, bv), wl.coo3_spec(dims, ci, cj, ck, cv)
    D = _dense3(dims, bi, bj, bk, bv) * _dense3(dims, ci, cj, ck, cv)
    both = (_dense3(dims, bi, bj, bk, np.ones(len(bv))) * _dense3(dims, ci, cj, ck, np.ones(len(cv)))) > 0
    (oi, oj, ok), v, _ = oracle.mul(b, c)
    lin = (oi.astype(np.int64) * 5 + oj) * 7 + ok
    assert 0 < len(lin) < min(len(bv), len(cv))
    assert np.all(np.diff(lin) > 0)                                   # ordered, unique
    assert np.array_equal(lin, np.flatnonzero(both.ravel()))          # exactly the intersection
    np.testing.assert_allclose(v, D[oi, oj, ok], rtol=0, atol=1e-15)
    # commutative
    (pi, pj, pk), pv, _ = oracle.mul(c, b)
    assert np.array_equal(pi, oi) and np.array_equal(pj, oj) and np.array_equal(pk, ok) and np.array_equal(pv, v)
    # B .* B squares the values on B's structure
    (qi, qj, qk), qv, _ = oracle.mul(b, b)
    assert np.array_equal(qi, bi) and np.array_equal(qj, bj) and np.array_equal(qk, bk) and np.array_equal(qv, bv * bv)
    # an explicit zero in one operand stays stored in the result
    z = bv.copy()
    z[::2] = 0.0
    (zi, _, _), zv, _ = oracle.mul(b, wl.coo3_spec(dims, bi, bj, bk, z))
    assert len(zi) == len(bv) and np.array_equal(zv, bv * z)
    # an empty operand, and operands with disjoint supports, give an empty result
    e = np.zeros(0, int)
    (ei, _, _), ev, _ = oracle.mul(b, wl.coo3_spec(dims, e, e, e, np.zeros(0)))
    assert len(ei) == 0 and len(ev) == 0
    even = wl.coo3_spec(dims, bi[bk % 2 == 0], bj[bk % 2 == 0], bk[bk % 2 == 0], bv[bk % 2 == 0])
    odd = wl.coo3_spec(dims, bi[bk % 2 == 1], bj[bk % 2 == 1], bk[bk % 2 == 1], bv[bk % 2 == 1])
    assert len(oracle.mul(even, odd)[1]) == 0
    # the sum over the product's entries is the inner product
    assert abs(v.sum() - oracle.innerprod(b, c)[0]) <= 1e-12 * np.abs(v).sum()
    # CSF operand walks to the same result
    (fi, fj, fk), fv, _ = oracle.mul(wl.csf3_from_sorted_coo(dims, bi, bj, bk, bv), c)
    assert np.array_equal(fi, oi) and np.array_equal(fk, ok) and np.array_equal(fv, v)


# ------------------------------------------------------------------ element-wise with a dense operand / result

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_mul_dense_vs_scipy_on_every_format(dtype):
    N, M = 37, 53
    r, c, v = wl.random_coo_entries(N, M, 400, seed=94, dtype=dtype)
    D = np.random.default_rng(95).uniform(-1, 1, (N, M)).astype(dtype)
    S = sp.coo_matrix((v.astype(np.float64), (r, c)), shape=(N, M)).tocsr().multiply(D.astype(np.float64)).tocsr()
    S.sort_indices()
    for spec in (wl.coo_spec(N, M, r, c, v), wl.csr_from_sorted_coo(N, M, r, c, v),
                 wl.dcsr_from_sorted_coo(N, M, r, c, v)):
        out = oracle.mul_dense(spec, D)                     # row-major storage order = scipy's sorted CSR
        np.testing.assert_allclose(out, S.data, rtol=0, atol=1e-15)
    # a column-major format: values come out in its own storage order
    csc = wl.csc_from_coo(N, M, r, c, v)
    coords, _ = oracle.to_coo(csc)
    np.testing.assert_allclose(oracle.mul_dense(csc, D), S.toarray()[coords[0], coords[1]], rtol=0, atol=1e-15)
    # ELL: padding positions give 0, the rest the products
    c3 = wl.config3(N=40, lo=0, hi=6, seed=96, dtype=dtype)
    ell = c3["ell"]
    D2 = np.random.default_rng(97).uniform(-1, 1, ell.dims).astype(dtype)
    out = oracle.mul_dense(ell, D2)
    crd = ell.levels[2].crd
    rows = np.tile(np.arange(40), len(crd) // 40)
    want = np.where(crd >= 0, ell.vals.astype(np.float64) * D2[rows, np.maximum(crd, 0)], 0.0)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-15)
    # D = 1 returns B's values, a non-square D of the transposed shape is refused
    assert np.array_equal(oracle.mul_dense(wl.coo_spec(N, M, r, c, v), np.ones((N, M), dtype)), v.astype(np.float64))
    with pytest.raises(TypeError):
        oracle.mul_dense(wl.coo_spec(N, M, r, c, v), D.T)


def test_add_to_dense_vs_numpy():
    N, M = 29, 31
    r1, c1, v1 = wl.random_coo_entries(N, M, 300, seed=98, dtype=np.float64)
    r2, c2, v2 = wl.random_coo_entries(N, M, 350, seed=99, dtype=np.float64)
    want = (sp.coo_matrix((v1, (r1, c1)), shape=(N, M)).toarray() + sp.coo_matrix((v2, (r2, c2)), shape=(N, M)).toarray())
    wmag = (sp.coo_matrix((np.abs(v1), (r1, c1)), shape=(N, M)).toarray() +
            sp.coo_matrix((np.abs(v2), (r2, c2)), shape=(N, M)).toarray())
    pairs = [(wl.csr_from_sorted_coo(N, M, r1, c1, v1), wl.coo_spec(N, M, r2, c2, v2)),   # the paper's CSR + COO
             (wl.coo_spec(N, M, r1, c1, v1), wl.csc_from_coo(N, M, r2, c2, v2)),
             (wl.dcsr_from_sorted_coo(N, M, r1, c1, v1), wl.csr_from_sorted_coo(N, M, r2, c2, v2))]
    for b, c in pairs:
        A, mag = oracle.add_to_dense(b, c)
        np.testing.assert_allclose(A, want, rtol=0, atol=1e-15)
        np.testing.assert_allclose(mag, wmag, rtol=0, atol=1e-15)
    # agrees with the sparse-result addition where that one stores an entry, 0 elsewhere
    (ri, ci), sv, _ = oracle.add(*pairs[0])
    A, _ = oracle.add_to_dense(*pairs[0])
    assert np.array_equal(A[ri, ci], sv)
    mask = np.ones((N, M), bool)
    mask[ri, ci] = False
    assert not A[mask].any()


# ------------------------------------------------------------------ packing into CSF / ELL / DIA

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_pack_csf_roundtrip_and_independent_builder(dtype):
    dims = (6, 5, 7)
    ci, cj, ck, v = wl.random_coo3_entries(dims, 120, seed=81, dtype=dtype, skew=1.5)
    perm = np.random.default_rng(0).permutation(len(v))                 # the packer orders the entries itself
    shuffled = wl.coo3_spec(dims, ci[perm], cj[perm], ck[perm], v[perm], ordered=False)
    pos0, crd0, pos1, crd1, pos2, crd2, vals = oracle.pack_csf(shuffled)
    # independent construction with numpy's unique
    assert np.array_equal(crd0, np.unique(ci))
    fib = np.unique(ci.astype(np.int64) * 5 + cj)
    assert np.array_equal(crd1, fib % 5) and len(crd1) == len(fib)
    assert list(pos0) == [0, len(crd0)] and pos1[-1] == len(crd1) and pos2[-1] == len(v)
    assert np.array_equal(np.diff(pos1), np.bincount(np.searchsorted(crd0, fib // 5), minlength=len(crd0)))
    assert np.array_equal(crd2, ck) and np.array_equal(vals, v.astype(np.float64))
    # walking the packed levels (Table 2 interpreter) gives back the sorted entries
    packed = wl.csf3_spec(dims, pos0, crd0, pos1, crd1, pos2, crd2, vals.astype(dtype))
    c, w = oracle.to_coo(packed)
    assert np.array_equal(c[0], ci) and np.array_equal(c[1], cj) and np.array_equal(c[2], ck)
    assert np.array_equal(w, v.astype(np.float64))
    # and the generator's own numpy builder agrees array by array
    ref = wl.csf3_from_sorted_coo(dims, ci, cj, ck, v)
    for lv, (p_, c_) in zip(ref.levels, ((pos0, crd0), (pos1, crd1), (pos2, crd2))):
        assert np.array_equal(lv.pos, p_) and np.array_equal(lv.crd, c_)
    e = np.zeros(0, int)
    out = oracle.pack_csf(wl.coo3_spec(dims, e, e, e, np.zeros(0, dtype)))
    assert list(out[0]) == [0, 0] and list(out[2]) == [0] and list(out[4]) == [0]


def test_pack_ell_vs_rows_and_roundtrip():
    N, M = 30, 40
    r, c, v = wl.random_coo_entries(N, M, 300, seed=82, dtype=np.float64)
    coo = wl.coo_spec(N, M, r, c, v)
    lens = np.bincount(r, minlength=N)
    W = int(lens.max())
    crd, vals, longest = oracle.pack_ell(coo, W)
    assert longest == W
    for i in range(N):                                                   # row by row, from the definition
        cols, vs = c[r == i], v[r == i]
        assert np.array_equal(crd[:len(cols), i], cols) and np.all(crd[len(cols):, i] == -1)
        assert np.array_equal(vals[:len(cols), i], vs) and np.all(vals[len(cols):, i] == 0)
    c2, w2 = oracle.to_coo(wl.ell_spec(N, M, crd, vals))                  # walk of the ELL levels
    order = np.lexsort((c2[1], c2[0]))
    assert np.array_equal(c2[0][order], r) and np.array_equal(c2[1][order], c) and np.array_equal(w2[order], v)
    x = wl.dense_vector(M, 5, np.float64)
    assert np.allclose(oracle.spmv(wl.ell_spec(N, M, crd, vals), x)[0], oracle.spmv(coo, x)[0], atol=1e-14)
    # too few slots: the tails of long rows are dropped, the longest row is still reported
    crd3, vals3, longest3 = oracle.pack_ell(coo, 3)
    assert longest3 == W and np.count_nonzero(crd3 >= 0) == int(np.minimum(lens, 3).sum())
    # CSR source walks to the same cells
    crd4, vals4, _ = oracle.pack_ell(wl.csr_from_sorted_coo(N, M, r, c, v), W)
    assert np.array_equal(crd4, crd) and np.array_equal(vals4, vals)


def test_pack_dia_vs_scipy():
    N, M = 25, 31
    rng = np.random.default_rng(83)
    offs = np.array([-20, -3, 0, 1, 7, 29])
    r, c = [], []
    for o in offs:                                                        # a banded matrix with holes
        i = np.arange(max(0, -o), min(N, M - o))
        i = i[rng.random(len(i)) < 0.7]
        r.append(i)
        c.append(i + o)
    r, c = np.concatenate(r), np.concatenate(c)
    order = np.lexsort((c, r))
    r, c = r[order], c[order]
    v = rng.uniform(-1, 1, len(r))
    coo = wl.coo_spec(N, M, r, c, v)
    offsets, vals = oracle.pack_dia(coo)
    assert np.array_equal(offsets, offs)
    D = sp.dia_matrix(sp.coo_matrix((v, (r, c)), shape=(N, M)))           # scipy: data[d, j] = A[j - off, j]
    so = np.argsort(D.offsets)
    assert np.array_equal(D.offsets[so], offsets)
    for d, o in enumerate(offsets):
        for i in range(N):
            j = i + o
            want = D.data[so[d], j] if 0 <= j < M and j < D.data.shape[1] else 0.0
            assert vals[d, i] == want
    c2, w2 = oracle.to_coo(wl.dia_spec(N, M, offsets, vals))              # walk of (dense, range, offset)
    dense = np.zeros((N, M))
    dense[c2[0], c2[1]] = w2
    assert np.array_equal(dense, sp.coo_matrix((v, (r, c)), shape=(N, M)).toarray())


def test_pack_hashed_rows_against_the_generators_tables_and_locate():
    """Table 3's hashed insert: the generator's independent Python insertion (same visiting order)
    builds the same tables; every stored coordinate is found by the hashed level's locate; the
    level walk returns exactly the entries; a full table reports what it had to drop."""
    N, M, W = 17, 40, 16
    r, c, v = wl.random_coo_entries(N, M, 120, seed=95, dtype=np.float64)
    coo = wl.coo_spec(N, M, r, c, v)
    crd, vals, dropped = oracle.pack_hashed_rows(coo, W)
    assert dropped == 0
    ref = wl.hashed_rows_from_coo(N, M, r, c, v, W)
    assert np.array_equal(crd.reshape(-1), ref.levels[1].crd) and np.array_equal(vals.reshape(-1), ref.vals)
    packed = wl.TensorSpec((N, M), ref.levels, vals.reshape(-1).copy())
    for i, j in zip(r, c):                                       # locate finds every inserted coordinate
        p, found = oracle.hashed_locate(packed.levels[1], int(i), int(j))
        assert found and crd.reshape(-1)[p] == j
    co, w = oracle.to_coo(packed)
    o = np.lexsort((co[1], co[0]))
    assert np.array_equal(co[0][o], r) and np.array_equal(co[1][o], c) and np.array_equal(w[o], v)
    # a row with more entries than slots: the surplus is reported, the table stays consistent
    rows = np.zeros(6, int)
    cols = np.array([0, 4, 8, 12, 16, 20])
    crd2, vals2, dropped2 = oracle.pack_hashed_rows(wl.coo_spec(2, 40, rows, cols, np.arange(6.0)), 4)
    assert dropped2 == 2 and np.count_nonzero(crd2 >= 0) == 4 and np.all(crd2[1] == -1)
