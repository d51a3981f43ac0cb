"""GPU parity at the benchmark's full sizes (same entry points and launch
configuration as bench.py): complete comparison where the oracle finishes in
seconds, otherwise sampled outputs computed by the oracle one by one plus
properties that hold at any size."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_coo_to_csr, gpu_mttkrp, gpu_spmv, gpu_ttv

pytestmark = pytest.mark.gpu


def test_config2_full_dia_and_csr():
    c2 = wl.config2(poison=True)
    ref, mag = oracle.spmv(c2["csr"], c2["x"])
    assert_close(gpu_spmv(c2["dia"], c2["x"]), ref, mag, np.float64, "c2 dia")
    assert_close(gpu_spmv(c2["csr"], c2["x"]), ref, mag, np.float64, "c2 csr")


def test_config3_full_ell_and_csr():
    c3 = wl.config3()
    ref, mag = oracle.spmv(c3["csr"], c3["x"])
    assert_close(gpu_spmv(c3["ell"], c3["x"]), ref, mag, np.float32, "c3 ell")
    assert_close(gpu_spmv(c3["csr"], c3["x"]), ref, mag, np.float32, "c3 csr")


def test_config4_full_pipelines():
    c4 = wl.config4(with_sorted=True)
    coo, x = c4["coo"], c4["x"]
    N = coo.dims[0]
    row, col, vals = coo.levels[0].crd, coo.levels[1].crd, coo.vals
    ref, mag = oracle.spmv(coo, x)                       # order-independent definition
    # (i) direct SpMV on the unsorted COO
    assert_close(gpu_spmv(coo, x), ref, mag, np.float64, "c4 unsorted coo")
    # (iii) conversion: properties at full size ...
    pos, crd, vout = gpu_coo_to_csr(coo, 0)
    assert np.array_equal(pos, np.concatenate([[0], np.cumsum(np.bincount(row, minlength=N))]))
    rows_out = np.repeat(np.arange(N, dtype=np.int64), np.diff(pos))
    key_out = rows_out * N + crd
    assert np.all(np.diff(key_out) > 0), "entries not strictly ascending in (row, col)"
    assert np.array_equal(key_out, np.sort(row.astype(np.int64) * N + col)), "coordinate multiset changed"
    # ... and sampled rows against the oracle's conversion of exactly those rows
    rng = np.random.default_rng(0)
    lens = np.diff(pos)
    sample = np.unique(np.concatenate([rng.integers(0, N, 200), np.argsort(lens)[-3:], [0, N - 1]]))
    pick = np.isin(row, sample)
    spos, scrd, svals, _ = oracle.coo_to_csr(N, row[pick], col[pick], vals[pick], 0)
    for r in sample:
        a, b = pos[r], pos[r + 1]
        assert np.array_equal(crd[a:b], scrd[spos[r]:spos[r + 1]]), f"row {r} columns"
        assert np.array_equal(vout[a:b], svals[spos[r]:spos[r + 1]]), f"row {r} values"
    # (ii) sorted COO and CSR SpMV on the generator's sorted layout of the same entries
    rs, cs, vs = c4["sorted"]
    assert_close(gpu_spmv(wl.coo_spec(N, N, rs, cs, vs), x), ref, mag, np.float64, "c4 sorted coo")
    assert_close(gpu_spmv(wl.csr_from_sorted_coo(N, N, rs, cs, vs), x), ref, mag, np.float64, "c4 csr")


def _sub(spec_arrays, mask, dims):
    ci, cj, ck, v = (a[mask] for a in spec_arrays)
    return wl.coo3_spec(dims, ci, cj, ck, v)


def test_config5_full_ttv_and_mttkrp_sampled():
    c5 = wl.config5()
    coo, csf = c5["coo"], c5["csf"]
    dims = coo.dims
    ci, cj, ck = (coo.levels[k].crd for k in range(3))
    arrays = (ci, cj, ck, coo.vals)
    # ---- TTV: structure at full size, values on sampled fibers
    oi, oj, ov, n = gpu_ttv(coo, c5["c"])
    fkey = ci.astype(np.int64) * dims[1] + cj
    head = np.ones(len(fkey), bool)
    head[1:] = fkey[1:] != fkey[:-1]
    assert n == int(head.sum()) == len(csf.levels[1].crd)
    assert np.array_equal(oi.astype(np.int64) * dims[1] + oj, fkey[head])
    _, _, cv, n2 = gpu_ttv(csf, c5["c"])
    assert n2 == n
    rng = np.random.default_rng(1)
    fib_id = np.cumsum(head) - 1
    sample = np.unique(np.concatenate([rng.integers(0, n, 3000), [0, n - 1]]))
    mask = np.isin(fib_id, sample)
    ri, rj, rv, rm = oracle.ttv(_sub(arrays, mask, dims), c5["c"])
    assert np.array_equal(ri, oi[sample]) and np.array_equal(rj, oj[sample])
    assert_close(ov[sample], rv, rm, np.float32, "c5 ttv coo (sampled fibers)")
    assert_close(cv[sample], rv, rm, np.float32, "c5 ttv csf (sampled fibers)")
    # ---- MTTKRP: sampled output rows, including the heavy slice 0
    Ac = gpu_mttkrp(coo, c5["C"], c5["D"])
    Af = gpu_mttkrp(csf, c5["C"], c5["D"])
    present = np.unique(ci)
    rows = np.unique(np.concatenate([[0, 1, 2, present[-1]], rng.choice(present, 40)]))
    mask = np.isin(ci, rows)
    ref, mag = oracle.mttkrp(_sub(arrays, mask, dims), c5["C"], c5["D"])
    assert_close(Ac[rows], ref[rows], mag[rows], np.float32, "c5 mttkrp coo (sampled rows)")
    assert_close(Af[rows], ref[rows], mag[rows], np.float32, "c5 mttkrp csf (sampled rows)")
    absent = np.setdiff1d(np.arange(dims[0]), present)
    assert not Ac[absent].any() and not Af[absent].any(), "rows without entries must be zero"
    assert np.all(np.isfinite(Ac)) and np.all(np.isfinite(Af))
