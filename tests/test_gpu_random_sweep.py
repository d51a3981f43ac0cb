"""GPU parity on seeded random shapes: every entry point against the oracle on inputs whose
dimensions, entry counts, skew and dtype are drawn per seed (small enough for the oracle, ragged
against every tile size by construction)."""
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import (assert_close, gpu_add, gpu_coo_to_csr, gpu_innerprod, gpu_mttkrp, gpu_spdm,
                      gpu_spmv, gpu_ttm, gpu_ttv)

pytestmark = pytest.mark.gpu

# SPT_SWEEP_SEEDS=a:b widens the sweep for a one-off soak of new kernels (default: 12 seeds)
_lo, _hi = (int(t) for t in os.environ.get("SPT_SWEEP_SEEDS", "0:12").split(":"))
SEEDS = list(range(_lo, _hi))
SCALE = int(os.environ.get("SPT_SWEEP_SCALE", "1"))   # multiplies the largest entry count drawn


def _draw_matrix(seed):
    rng = np.random.default_rng(10_000 + seed)
    dtype = [np.float32, np.float64][seed % 2]
    side = int(6000 * SCALE ** 0.5)
    N, M = int(rng.integers(1, side)), int(rng.integers(1, side))
    nnz = int(rng.integers(0, min(N * M, 60_000 * SCALE) + 1))
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=20_000 + seed, dtype=dtype)
    if seed % 3 == 0 and len(r) > 10:                       # a few heavy rows
        heavy = rng.integers(0, N, 3)
        r[rng.random(len(r)) < 0.4] = heavy[0]
        order = np.lexsort((c, r))
        key, first = np.unique(r[order].astype(np.int64) * M + c[order], return_index=True)
        r, c, v = r[order][first], c[order][first], v[order][first]
    return N, M, r, c, v, dtype


@pytest.mark.parametrize("seed", SEEDS)
def test_matrix_kernels(seed):
    N, M, r, c, v, dtype = _draw_matrix(seed)
    x = wl.dense_vector(M, seed, dtype)
    coo = wl.coo_spec(N, M, r, c, v)
    ref, mag = oracle.spmv(coo, x)
    csr = wl.csr_from_sorted_coo(N, M, r, c, v)
    hinted = wl.csr_from_sorted_coo(N, M, r, c, v)
    hinted.levels[1].max_children = 8                       # may be violated: must stay correct
    rng = np.random.default_rng(seed)
    perm = rng.permutation(len(v))
    shuffled = wl.coo_spec(N, M, r[perm], c[perm], v[perm], ordered=False)
    for name, spec in (("coo", coo), ("csr", csr), ("csr hinted", hinted), ("coo unordered", shuffled),
                       ("dcsr", wl.dcsr_from_sorted_coo(N, M, r, c, v)), ("csc", wl.csc_from_coo(N, M, r, c, v))):
        assert_close(gpu_spmv(spec, x), ref, mag, dtype, f"seed {seed} spmv {name}")
    for order in (0, 1):
        pos, crd, vals = gpu_coo_to_csr(shuffled, order)
        rpos, rcrd, rvals, _ = oracle.coo_to_csr(N, r[perm], c[perm], v[perm], order)
        assert np.array_equal(pos, rpos) and np.array_equal(crd, rcrd) and np.array_equal(vals, rvals)
    J = int(rng.integers(1, 70))
    Cm = rng.uniform(-1, 1, (M, J)).astype(dtype)
    A, Amag = oracle.spdm(coo, Cm)
    assert_close(gpu_spdm(coo, Cm), A, Amag, dtype, f"seed {seed} spdm J={J}")
    r2, c2, v2 = wl.random_coo_entries(N, M, int(rng.integers(0, min(N * M, 40_000 * SCALE) + 1)),
                                       seed=30_000 + seed, dtype=dtype)
    other = wl.coo_spec(N, M, r2, c2, v2)
    (ri, ci), rv, rm = oracle.add(coo, other)
    idx, gv = gpu_add(coo, other, "coo")
    assert np.array_equal(idx[0], ri) and np.array_equal(idx[1], ci)
    assert_close(gv, rv, rm, dtype, f"seed {seed} add coo")
    (pos, cols), gv = gpu_add(csr, wl.csr_from_sorted_coo(N, M, r2, c2, v2), "csr")
    assert np.array_equal(pos, np.concatenate([[0], np.cumsum(np.bincount(ri, minlength=N))]))
    assert np.array_equal(cols, ci)
    a, m = oracle.innerprod(coo, other)
    assert_close(gpu_innerprod(coo, other), a, m, dtype, f"seed {seed} innerprod matrices")
    # element-wise product, CSR x COO (result CSR) and COO x CSR (result COO)
    (ri, ci), rv, rm = oracle.mul(csr, other)
    (pos, cols), gv = gpu_add(csr, other, "csr", op="mul")
    assert np.array_equal(pos, np.concatenate([[0], np.cumsum(np.bincount(ri, minlength=N))]))
    assert np.array_equal(cols, ci)
    assert_close(gv, rv, rm, dtype, f"seed {seed} mul csr x coo")
    idx, gv = gpu_add(other, csr, "coo", op="mul")
    assert np.array_equal(idx[0], ri) and np.array_equal(idx[1], ci)
    assert_close(gv, rv, rm, dtype, f"seed {seed} mul coo x csr")
    # the same matrix blocked: BCSR (own kernel) and CSB (per-value path), block shape per seed
    b1, b2 = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    xb = wl.dense_vector(-(-M // b2) * b2, seed + 100, dtype)
    for name, spec in (("bcsr", wl.bcsr_from_coo(N, M, r, c, v, b1, b2)),
                       ("csb", wl.csb_from_coo(N, M, r, c, v, b1, b2))):
        if name == "csb" and (-(-N // b1)) * (-(-M // b2)) > 4_000_000:
            continue                                        # CSB keeps one pos entry per block of the grid
        bref, bmag = oracle.spmv_blocked(spec, xb)
        assert_close(gpu_spmv(spec, xb), bref, bmag, dtype, f"seed {seed} spmv {name} {b1}x{b2}")


@pytest.mark.parametrize("seed", SEEDS)
def test_tensor_kernels(seed):
    rng = np.random.default_rng(40_000 + seed)
    dtype = [np.float64, np.float32][seed % 2]
    dims = tuple(int(d) for d in rng.integers(1, int(120 * SCALE ** (1 / 3)), 3))
    cells = dims[0] * dims[1] * dims[2]
    nnz = int(rng.integers(0, min(cells, 50_000 * SCALE) + 1))
    skew = [None, 1.2, 2.0][seed % 3]
    ci, cj, ck, v = wl.random_coo3_entries(dims, nnz, 50_000 + seed, dtype=dtype, dist="u11", skew=skew)
    coo = wl.coo3_spec(dims, ci, cj, ck, v)
    csf = wl.csf3_from_sorted_coo(dims, ci, cj, ck, v)
    c = wl.dense_vector(dims[2], seed, dtype)
    ti, tj, tv, tm = oracle.ttv(coo, c)
    gi, gj, gv, n = gpu_ttv(coo, c)
    assert n == len(ti) and np.array_equal(gi, ti) and np.array_equal(gj, tj)
    assert_close(gv, tv, tm, dtype, f"seed {seed} ttv coo")
    assert_close(gpu_ttv(csf, c)[2], tv, tm, dtype, f"seed {seed} ttv csf")
    J = int(rng.integers(1, 70))
    Cm = rng.uniform(-1, 1, (dims[1], J)).astype(dtype)
    Dm = rng.uniform(-1, 1, (dims[2], J)).astype(dtype)
    A, Amag = oracle.mttkrp(coo, Cm, Dm)
    assert_close(gpu_mttkrp(coo, Cm, Dm), A, Amag, dtype, f"seed {seed} mttkrp coo J={J}")
    assert_close(gpu_mttkrp(csf, Cm, Dm), A, Amag, dtype, f"seed {seed} mttkrp csf J={J}")
    K = int(rng.integers(1, 40))
    Ck = rng.uniform(-1, 1, (K, dims[2])).astype(dtype)
    mi, mj, mv, mm = oracle.ttm(coo, Ck)
    qi, qj, qv = gpu_ttm(coo, Ck)
    assert np.array_equal(qi, mi) and np.array_equal(qj, mj)
    assert_close(qv, mv, mm, dtype, f"seed {seed} ttm coo K={K}")
    assert_close(gpu_ttm(csf, Ck, is_csf=True)[2], mv, mm, dtype, f"seed {seed} ttm csf K={K}")
    oi, oj, ok, ov = wl.random_coo3_entries(dims, int(rng.integers(0, min(cells, 30_000 * SCALE) + 1)),
                                            60_000 + seed, dtype=dtype, dist="u11")
    other = wl.coo3_spec(dims, oi, oj, ok, ov)
    a, m = oracle.innerprod(coo, other)
    assert_close(gpu_innerprod(coo, other), a, m, dtype, f"seed {seed} innerprod")
    (ri, rj, rk), rv, rm = oracle.add(coo, other)
    idx, pv = gpu_add(coo, other, "coo3")
    assert np.array_equal(idx[0], ri) and np.array_equal(idx[1], rj) and np.array_equal(idx[2], rk)
    assert_close(pv, rv, rm, dtype, f"seed {seed} plus")
    (ri, rj, rk), rv, rm = oracle.mul(coo, other)
    idx, pv = gpu_add(coo, other, "coo3", op="mul")
    assert np.array_equal(idx[0], ri) and np.array_equal(idx[1], rj) and np.array_equal(idx[2], rk)
    assert_close(pv, rv, rm, dtype, f"seed {seed} element-wise product")
