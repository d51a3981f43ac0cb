"""GPU parity: spt_spmv through the C ABI vs the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_spmv

pytestmark = pytest.mark.gpu

CHUNK = 2048  # entries per workgroup of the CSR/COO kernel: sizes below straddle it


def _check(spec, x, what):
    ref, mag = oracle.spmv(spec, x)
    got = gpu_spmv(spec, x)
    assert_close(got, ref, mag, spec.vals.dtype, what)
    return got


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("nnz", [0, 1, 63, 64, 65, 2047, 2048, 2049, 4096, 5000, 70001])
def test_csr_coo_random_sizes(dtype, nnz):
    N, M = 997, 1201
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=100 + nnz, dtype=dtype)
    x = wl.dense_vector(M, 7, dtype)
    _check(wl.csr_from_sorted_coo(N, M, r, c, v), x, f"csr nnz={nnz}")
    _check(wl.coo_spec(N, M, r, c, v), x, f"coo nnz={nnz}")
    p = np.random.default_rng(1).permutation(len(v))
    _check(wl.coo_spec(N, M, r[p], c[p], v[p], ordered=False), x, f"coo-unsorted nnz={nnz}")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_csr_coo_degenerate_structures(dtype):
    x = wl.dense_vector(50, 3, dtype)
    # one row holds everything (spans several chunks), all other rows empty
    n = 3 * CHUNK + 17
    rng = np.random.default_rng(5)
    c = rng.integers(0, 50, n)
    v = rng.uniform(-1, 1, n).astype(dtype)
    for row in (0, 5, 9):
        r = np.full(n, row)
        _check(wl.csr_from_sorted_coo(10, 50, r, c, v), x, f"csr single row {row}")
        _check(wl.coo_spec(10, 50, r, c, v), x, f"coo single row {row}")
    # many empty rows between few entries, rows >> entries
    r = np.array([3, 3, 40000, 99999])
    c4 = np.array([1, 2, 3, 4])
    v4 = np.array([1, 2, 3, 4], dtype)
    _check(wl.csr_from_sorted_coo(100000, 50, r, c4, v4), x, "csr mostly empty")
    _check(wl.coo_spec(100000, 50, r, c4, v4), x, "coo mostly empty")
    # more than 2^20 rows: few entries still take the chunked kernel (fill + carries)
    _check(wl.coo_spec(3_000_000, 50, np.array([3, 3, 40000, 2_999_999]), c4, v4), x, "coo, 3M rows, 4 entries")
    # row boundaries exactly on chunk boundaries
    r = np.repeat(np.arange(4), CHUNK)
    c = rng.integers(0, 50, 4 * CHUNK)
    v = rng.uniform(-1, 1, 4 * CHUNK).astype(dtype)
    _check(wl.csr_from_sorted_coo(4, 50, r, c, v), x, "csr aligned rows")
    _check(wl.coo_spec(4, 50, r, c, v), x, "coo aligned rows")
    # duplicates are summed by SpMV
    r, c, v = wl.random_coo_entries(20, 50, 6000, seed=8, dtype=dtype, duplicates=True)
    _check(wl.csr_from_sorted_coo(20, 50, r, c, v), x, "csr duplicates")
    _check(wl.coo_spec(20, 50, r, c, v), x, "coo duplicates")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("nnz", [255, 257, 1023, 65_535, 65_536, 65_537, 200_000])
def test_sorted_coo_on_both_sides_of_the_single_launch_limit(dtype, nnz):
    """Up to 65 536 entries sorted COO runs in one launch (a wave per 256 entries, the owner of
    a row reads on past its piece); above, the chunked kernel with carries. Rows of 1 to 3000
    entries, runs of empty rows, the last rows empty, an infinite x value under the last entry."""
    N, M = 9000, 700
    rng = np.random.default_rng(nnz)
    lens = np.minimum(rng.zipf(1.4, 4000), min(3000, nnz // 3))
    lens = lens[np.cumsum(lens) <= nnz]
    rows = np.sort(rng.choice(N - 50, len(lens), replace=False))      # the last 50 rows stay empty
    r = np.repeat(rows, lens)
    r = np.concatenate([r, np.full(nnz - len(r), rows[-1] + 1)])      # fill up with one more long row
    c = rng.integers(0, M, nnz)
    c = c[np.lexsort((c, r))]                                         # columns ascend inside every row
    v = rng.uniform(-1, 1, nnz).astype(dtype)
    x = wl.dense_vector(M, 11, dtype)
    _check(wl.coo_spec(N, M, r, c, v), x, f"sorted coo nnz={nnz}")
    x2 = x.copy()
    x2[c[-1]] = np.inf
    v[c == c[-1]] = 1.0
    spec = wl.coo_spec(N, M, r, c, v)
    ref, _ = oracle.spmv(spec, x2)
    got = gpu_spmv(spec, x2)
    assert np.array_equal(np.isinf(got), np.isinf(ref)) and not np.isnan(got).any()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_buffers_that_are_not_16_byte_aligned(dtype):
    """Arrays one element past an aligned address take the scalar-load paths."""
    N, M = 1000, 1200
    r, c, v = wl.random_coo_entries(N, M, 9000, seed=77, dtype=dtype)
    x = wl.dense_vector(M, 7, dtype)
    c2 = wl.config2(N=1000, dtype=dtype)
    c3 = wl.config3(N=1000, dtype=dtype)
    for spec, xx in ((wl.csr_from_sorted_coo(N, M, r, c, v), x), (wl.coo_spec(N, M, r, c, v), x),
                     (c2["dia"], c2["x"]), (c3["ell"], c3["x"])):
        ref, mag = oracle.spmv(spec, xx)
        assert_close(gpu_spmv(spec, xx, misalign=True), ref, mag, dtype, spec.name + " misaligned")


def test_config1_full_and_deterministic():
    c1 = wl.config1()
    for fmt in ("csr", "coo"):
        ref, mag = oracle.spmv(c1[fmt], c1["x"])
        a, b = gpu_spmv(c1[fmt], c1["x"], repeat=2)
        assert_close(a, ref, mag, np.float64, f"c1 {fmt}")
        assert np.array_equal(a, b), "run-to-run bits differ"


def test_power_law_rows_scaled_config4():
    c4 = wl.config4(N=40_000, nnz_target=600_000, max_row=20_000)
    coo = c4["coo"]
    r, c = coo.levels[0].crd, coo.levels[1].crd
    _check(coo, c4["x"], "c4 unsorted coo")
    o = np.lexsort((c, r))
    rs, cs, vs = r[o], c[o], coo.vals[o]
    a = _check(wl.coo_spec(40_000, 40_000, rs, cs, vs), c4["x"], "c4 sorted coo")
    csr = wl.csr_from_sorted_coo(40_000, 40_000, rs, cs, vs)
    b = _check(csr, c4["x"], "c4 csr, kernel chosen by the mean row length")
    lv = csr.levels[1]
    _check(wl.csr_spec(40_000, 40_000, lv.pos, lv.crd, csr.vals, max_row=20_000), c4["x"],
           "c4 csr, declared long rows: entry-balanced kernel")
    assert np.bincount(r).max() > 2 * CHUNK      # a row really spans several chunks


@pytest.mark.parametrize("dtype,N", [(np.float64, 6_000_000), (np.float32, 20_000_000)])
def test_unordered_coo_with_more_rows_than_one_lds_window(dtype, N):
    """Row count so large that a bin's rows need several LDS sub-ranges, and a row so long
    that its bin is cut into several slices (slices combine with atomics)."""
    rng = np.random.default_rng(4)
    n = 700_000
    row = rng.integers(0, N, n)
    row[: n // 2] = N - 7                       # one heavy row: > 262144 entries in one bin
    col = rng.integers(0, 1000, n)
    v = rng.uniform(-1, 1, n).astype(dtype)
    p = rng.permutation(n)
    spec = wl.coo_spec(N, 1000, row[p], col[p], v[p], ordered=False)
    x = wl.dense_vector(1000, 5, dtype)
    _check(spec, x, f"unordered coo N={N}")


def test_exact_integer_data_is_bit_exact():
    N, M = 3000, 2000
    r, c, v = wl.random_coo_entries(N, M, 50_000, seed=9, dtype=np.float32, dist="int")
    x = wl.dense_vector(M, 10, np.float32, "int")
    ref, _ = oracle.spmv(wl.coo_spec(N, M, r, c, v), x)
    for spec in (wl.csr_from_sorted_coo(N, M, r, c, v), wl.coo_spec(N, M, r, c, v),
                 wl.coo_spec(N, M, r[::-1].copy(), c[::-1].copy(), v[::-1].copy(), ordered=False)):
        assert np.array_equal(gpu_spmv(spec, x).astype(np.float64), ref)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N", [1, 255, 256, 257, 100_003])
def test_dia_scaled_config2_with_poison(dtype, N):
    c2 = wl.config2(N=max(N, 8), poison=True, dtype=dtype)
    got = _check(c2["dia"], c2["x"], f"dia N={N}")
    assert np.isfinite(got).all()
    _check(c2["csr"], c2["x"], f"c2 csr N={N}")


def test_dia_rectangular_and_outside_diagonals():
    rng = np.random.default_rng(3)
    for (N, M) in ((700, 1000), (1000, 700)):
        off = np.array([-1200, -699, -3, 0, 1, 250, 999, 5000])
        diag = rng.uniform(-1, 1, (len(off), N))
        i = np.arange(N)
        for d, o in enumerate(off):
            diag[d, ~((i + o >= 0) & (i + o < M))] = np.nan
        _check(wl.dia_spec(N, M, off, diag), wl.dense_vector(M, 4), f"dia {N}x{M}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("N", [1, 300, 100_001])
def test_ell_scaled_config3_with_poisoned_padding(dtype, N):
    c3 = wl.config3(N=max(N, 40), dtype=dtype)
    ell = c3["ell"]
    v = ell.vals.copy()
    v[ell.levels[2].crd < 0] = np.nan
    got = _check(wl.TensorSpec(ell.dims, ell.levels, v), c3["x"], f"ell N={N}")
    assert np.isfinite(got).all()
    _check(c3["csr"], c3["x"], f"c3 csr N={N}")
    # a matrix whose rows are all empty: every slot is padding
    z = wl.config3(N=50, lo=0, hi=0, dtype=dtype)
    assert z["W"] == 0 or np.all(z["ell"].levels[2].crd < 0)
    _check(z["ell"], z["x"], "ell all padding")


def _with_hint(spec, bound):
    lv = spec.levels[1]
    return wl.csr_spec(spec.dims[0], spec.dims[1], lv.pos, lv.crd, spec.vals, max_row=bound)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("lo,hi", [(0, 3), (1, 7), (0, 12), (9, 16), (8, 32)])
def test_csr_kernel_choice_by_mean_row_length_and_by_hint(dtype, lo, hi):
    """Plain (pos, crd) CSR with a short mean row runs the streamed kernel (256 rows' entries
    through LDS, one lane per row) with no hint at all; a declared bound <= 32 selects the same
    kernel (same bits), a larger one the entry-balanced kernel; all match the oracle."""
    c3 = wl.config3(N=5003, lo=lo, hi=hi, dtype=dtype)
    hinted = c3["csr"]
    assert hinted.levels[1].max_children == c3["W"] <= 32
    plain = _with_hint(hinted, 0)
    ref, mag = oracle.spmv(hinted, c3["x"])
    a, b = gpu_spmv(plain, c3["x"], repeat=2)
    assert_close(a, ref, mag, dtype, f"no hint, rows {lo}..{hi}")
    assert np.array_equal(a, b), "run-to-run bits differ"
    assert np.array_equal(gpu_spmv(hinted, c3["x"]), a), "the hint selects the same kernel"
    assert_close(gpu_spmv(_with_hint(hinted, 100_000), c3["x"]), ref, mag, dtype,
                 f"entry-balanced kernel rows {lo}..{hi}")
    assert_close(gpu_spmv(plain, c3["x"], misalign=True), ref, mag, dtype, "streamed kernel, unaligned")


@pytest.mark.parametrize("which", ["c2", "c3"])
def test_unhinted_csr_of_configs_2_and_3_is_bit_reproducible(which):
    cfg = wl.config2(N=300_001) if which == "c2" else wl.config3(N=100_003)
    plain = _with_hint(cfg["csr"], 0)
    dt = plain.vals.dtype
    ref, mag = oracle.spmv(plain, cfg["x"])
    a, b = gpu_spmv(plain, cfg["x"], repeat=2)
    assert_close(a, ref, mag, dt, f"unhinted {which} csr")
    assert np.array_equal(a, b)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("nnz_mod", [0, 1, 2, 3])
def test_streamed_kernel_with_long_rows_among_short_ones(dtype, nnz_mod):
    """Mean row length 8, so the streamed kernel runs, but single rows hold 60, 3000, 9000 and
    40 000 entries: parts of a row longer than 48 products are added up by the whole wave, whole
    LDS pieces inside one row are added up in registers. The entry count takes every remainder
    modulo 4 (the last 16-byte group of the arrays is partial)."""
    N, M = 12_000, 50_000
    r, c, v = wl.random_coo_entries(N, M, 40_000 + nnz_mod, seed=70 + nnz_mod, dtype=dtype)
    rng = np.random.default_rng(71)
    rows, cols, vals = [r], [c], [v]
    for row, n in ((3, 60), (700, 3000), (701, 9000), (5000, 40_000), (N - 1, 5000)):
        keep = rows[0] != row
        rows[0], cols[0], vals[0] = rows[0][keep], cols[0][keep], vals[0][keep]
        rows.append(np.full(n, row))
        cols.append(np.sort(rng.choice(M, n, replace=False)))
        vals.append(rng.uniform(-1, 1, n).astype(dtype))
    r, c, v = np.concatenate(rows), np.concatenate(cols), np.concatenate(vals)
    r, c, v = r[: len(r) - (len(r) - nnz_mod) % 4], c[: len(r) - (len(r) - nnz_mod) % 4], v[: len(r) - (len(r) - nnz_mod) % 4]
    order = np.lexsort((c, r))
    spec = wl.csr_from_sorted_coo(N, M, r[order], c[order], v[order])
    assert len(spec.vals) % 4 == nnz_mod and len(spec.vals) <= 32 * N
    x = wl.dense_vector(M, 72, dtype)
    ref, mag = oracle.spmv(spec, x)
    a, b = gpu_spmv(spec, x, repeat=2)
    assert_close(a, ref, mag, dtype, "long rows, streamed")
    assert np.array_equal(a, b)
    assert_close(gpu_spmv(spec, x, misalign=True), ref, mag, dtype, "long rows, streamed, unaligned")
    assert_close(gpu_spmv(_with_hint(spec, 40_000), x), ref, mag, dtype, "long rows, entry-balanced")


@pytest.mark.parametrize("heavy_row", [0, 150_000])
def test_large_unhinted_csr_picks_its_kernel_on_the_device(heavy_row):
    """From 2^25 entries on, a CSR matrix without a declared row bound has the entry counts of
    its 256-row blocks inspected on the device: even blocks keep the streamed kernel (same bits
    as with a declared bound of 16), one block holding a 150 000-entry row switches to the
    entry-balanced kernel (same bits as with a declared bound of 150 000)."""
    N = M = 2_100_000
    K = 16
    rng = np.random.default_rng(90 + (heavy_row > 0))
    cols = (rng.integers(0, M, N, dtype=np.int64)[:, None] + np.arange(K, dtype=np.int64)[None, :] * 131_071) % M
    cols.sort(axis=1)
    lens = np.full(N, K, dtype=np.int64)
    crd = cols.reshape(-1)
    if heavy_row:
        at = 1_234_567
        extra = np.sort(rng.choice(M, heavy_row, replace=False))
        crd = np.concatenate([crd[: at * K], extra, crd[(at + 1) * K:]])
        lens[at] = heavy_row
    del cols
    pos = np.concatenate([[0], np.cumsum(lens)])
    nnz = int(pos[-1])
    assert nnz >= 2**25 and nnz <= 32 * N
    vals = rng.uniform(-1, 1, nnz).astype(np.float32)
    plain = wl.csr_spec(N, M, pos, crd, vals)
    x = wl.dense_vector(M, 92, np.float32)
    ref, mag = oracle.spmv(plain, x)
    a, b = gpu_spmv(plain, x, repeat=2)
    assert_close(a, ref, mag, np.float32, f"large unhinted csr, heavy row {heavy_row}")
    assert np.array_equal(a, b), "run-to-run bits differ"
    same = gpu_spmv(_with_hint(plain, heavy_row if heavy_row else K), x)
    assert np.array_equal(a, same), "the device-side choice differs from the expected kernel"
    other = gpu_spmv(_with_hint(plain, K if heavy_row else 100_000), x)
    assert_close(other, ref, mag, np.float32, "the kernel not chosen")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_csr_hint_that_the_data_violates_stays_correct(dtype):
    """A declared bound of 8 on a matrix with one row of 9000 entries: the streamed kernel takes
    the long row in several LDS pieces; slower, never wrong."""
    N, M = 3000, 10_000
    r, c, v = wl.random_coo_entries(N, M, 20_000, seed=77, dtype=dtype)
    rng = np.random.default_rng(78)
    long_cols = np.sort(rng.choice(M, 9000, replace=False))
    keep = r != 7
    r = np.concatenate([r[keep], np.full(9000, 7)])
    c = np.concatenate([c[keep], long_cols])
    v = np.concatenate([v[keep], rng.uniform(-1, 1, 9000).astype(dtype)])
    order = np.lexsort((c, r))
    lying = wl.csr_from_sorted_coo(N, M, r[order], c[order], v[order])
    lying.levels[1].max_children = 8
    x = wl.dense_vector(M, 79, dtype)
    ref, mag = oracle.spmv(lying, x)
    assert_close(gpu_spmv(lying, x), ref, mag, dtype, "violated hint")


def test_unsupported_and_invalid_descriptors_report_errors():
    import paper_1804_10112_amd as spt
    import torch
    c1 = wl.config1(N=64, nnz=100)
    c1["csr"].levels[1].max_children = 5000     # declared long rows: the kernel that needs a workspace
    A = spt.DeviceTensor(c1["csr"])
    x = torch.zeros(64, dtype=torch.float64, device="cuda")
    y = torch.zeros(64, dtype=torch.float64, device="cuda")
    with pytest.raises(spt.SptError) as e:
        spt.spt_spmv(A, x, y, None)          # workspace missing
    assert e.value.status == 3
    with pytest.raises(spt.SptError) as e:
        spt.spt_spmv(A, None, y, A.workspace(spt.SPT_OP_SPMV))
    assert e.value.status == 1
