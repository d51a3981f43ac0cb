"""GPU parity at the benchmark's full sizes (same entry points and launch
configuration as bench.py): every output element against the oracle."""
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
    # ... every column and every value against numpy's sort of the same keys (keys are unique)
    order = np.argsort(row.astype(np.int64) * N + col, kind="stable")
    assert np.array_equal(crd, col[order]), "columns differ from the sorted input"
    assert np.array_equal(vout, vals[order]), "values differ from the sorted input"
    del order, key_out, rows_out
    # ... and every output array against the oracle's conversion (Table 3's append sequence after
    # its own merge sort)
    opos, ocrd, ovals, _ = oracle.coo_to_csr(N, row, col, vals, 0)
    assert np.array_equal(pos, opos) and np.array_equal(crd, ocrd) and np.array_equal(vout, ovals)
    del opos, ocrd, ovals
    # (ii) sorted COO and CSR SpMV on the generator's sorted layout of the same entries
    rs, cs, vs = c4["sorted"]
    assert_close(gpu_spmv(wl.coo_spec(N, N, rs, cs, vs), x), ref, mag, np.float64, "c4 sorted coo")
    assert_close(gpu_spmv(wl.csr_from_sorted_coo(N, N, rs, cs, vs), x), ref, mag, np.float64, "c4 csr")


def test_config5_full_ttv_and_mttkrp():
    """Every fibre of TTV and every row of MTTKRP against the oracle's definitions at full size
    (the oracle needs about ten seconds for each)."""
    c5 = wl.config5()
    coo, csf = c5["coo"], c5["csf"]
    dims = coo.dims
    # ---- TTV
    ri, rj, rv, rm = oracle.ttv(coo, c5["c"])
    oi, oj, ov, n = gpu_ttv(coo, c5["c"])
    assert n == len(ri) == len(csf.levels[1].crd)
    assert np.array_equal(oi, ri) and np.array_equal(oj, rj), "fibre coordinates"
    assert_close(ov, rv, rm, np.float32, "c5 ttv coo")
    _, _, cv, n2 = gpu_ttv(csf, c5["c"])
    assert n2 == n
    assert_close(cv, rv, rm, np.float32, "c5 ttv csf")
    del ri, rj, rv, rm, oi, oj, ov, cv
    # ---- MTTKRP, all rows, against the unfactored definition
    ref, mag = oracle.mttkrp(coo, c5["C"], c5["D"])
    Ac = gpu_mttkrp(coo, c5["C"], c5["D"])
    assert_close(Ac, ref, mag, np.float32, "c5 mttkrp coo")
    Af = gpu_mttkrp(csf, c5["C"], c5["D"])
    assert_close(Af, ref, mag, np.float32, "c5 mttkrp csf")
    absent = np.setdiff1d(np.arange(dims[0]), np.unique(coo.levels[0].crd))
    assert len(absent) > 0 and not Ac[absent].any() and not Af[absent].any(), "rows without entries must be zero"
