"""GPU parity: spt_coo_to_csr vs the oracle -- every output bit-exact."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import gpu_coo_to_csr

pytestmark = pytest.mark.gpu

TILE = 4096  # records per workgroup of the radix sort: sizes below straddle it


def _check(N, M, r, c, v, order, ordered=False, what=""):
    spec = wl.coo_spec(N, M, r, c, v, ordered=ordered)
    pos, crd, vout = gpu_coo_to_csr(spec, order)
    rpos, rcrd, rv, _ = oracle.coo_to_csr(N, r, c, v, order)
    assert np.array_equal(pos, rpos), f"{what}: pos differs"
    assert np.array_equal(crd, rcrd), f"{what}: crd differs"
    assert np.array_equal(vout.view(np.uint8), rv.view(np.uint8)), f"{what}: vals differ"
    assert pos[0] == 0 and pos[-1] == len(v) and np.all(np.diff(pos) >= 0)


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("nnz", [0, 1, 255, 256, 4095, 4096, 4097, 3 * 4096 + 5, 100_003])
def test_random_unsorted(order, dtype, nnz):
    N, M = 1500, 70_000                      # 11 row bits (2 passes), 17 col bits (3 passes)
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=200 + nnz, dtype=dtype, sort=False)
    _check(N, M, r, c, v, order, what=f"nnz={nnz}")


@pytest.mark.parametrize("order", [0, 1])
def test_duplicates_keep_input_order(order):
    N, M = 37, 19
    r, c, v = wl.random_coo_entries(N, M, 20_000, seed=5, duplicates=True, sort=False)
    v = np.arange(len(v), dtype=np.float64)   # values identify the input position
    _check(N, M, r, c, v, order, what="duplicates")


@pytest.mark.parametrize("order", [0, 1])
def test_degenerate_shapes(order):
    rng = np.random.default_rng(1)
    n = 2 * TILE + 9
    v = rng.uniform(-1, 1, n)
    _check(1, 1, np.zeros(n, int), np.zeros(n, int), v, order, what="1x1")
    _check(1, 300, np.zeros(n, int), rng.integers(0, 300, n), v, order, what="one row")
    _check(300, 1, rng.integers(0, 300, n), np.zeros(n, int), v, order, what="one col")
    _check(100_000, 3, np.array([99_999, 0, 50_000, 0]), np.array([2, 1, 0, 0]),
           np.array([1., 2., 3., 4.]), order, what="rows >> entries")
    # runs of empty rows of every length next to a dense cluster (long runs are written by a whole wave)
    rr = np.concatenate([rng.integers(0, 1_000_000, 5000), rng.integers(400_000, 400_300, 6000)])
    _check(1_000_000, 50, rr, rng.integers(0, 50, rr.size), rng.uniform(-1, 1, rr.size), order,
           what="sparse rows with a dense cluster")
    big = 2**31 - 10                           # maximum dimension sizes: all 31 key bits used
    r = np.array([big - 1, 0, big - 1, 12345, 2**30])
    c = np.array([big - 2, 5, 0, 2**30 + 1, 7])
    spec = wl.coo_spec(5, big, [0, 1, 2, 3, 4], c, np.arange(5.0), ordered=False)
    pos, crd, vout = gpu_coo_to_csr(spec, order)
    assert list(pos) == [0, 1, 2, 3, 4, 5] and np.array_equal(crd, c)


@pytest.mark.parametrize("order", [0, 1])
def test_buffers_that_are_not_16_byte_aligned(order):
    N, M = 700, 900
    r, c, v = wl.random_coo_entries(N, M, 20_000, seed=12, sort=False)
    spec = wl.coo_spec(N, M, r, c, v, ordered=False)
    pos, crd, vout = gpu_coo_to_csr(spec, order, misalign=True)
    rpos, rcrd, rv, _ = oracle.coo_to_csr(N, r, c, v, order)
    assert np.array_equal(pos, rpos) and np.array_equal(crd, rcrd) and np.array_equal(vout, rv)


def test_sorted_flagged_input_skips_the_sort():
    N, M = 800, 900
    r, c, v = wl.random_coo_entries(N, M, 30_000, seed=6)
    _check(N, M, r, c, v, 0, ordered=True, what="flagged sorted")
    _check(N, M, r, c, v, 1, ordered=True, what="flagged sorted, stable")


def test_csr_to_coo_to_csr_is_a_fixed_point():
    N, M = 500, 600
    r, c, v = wl.random_coo_entries(N, M, 9000, seed=7, sort=False)
    pos, crd, vout = gpu_coo_to_csr(wl.coo_spec(N, M, r, c, v, ordered=False), 0)
    rows = np.repeat(np.arange(N), np.diff(pos))
    pos2, crd2, v2 = gpu_coo_to_csr(wl.coo_spec(N, M, rows, crd, vout, ordered=False), 0)
    assert np.array_equal(pos, pos2) and np.array_equal(crd, crd2) and np.array_equal(vout, v2)
    # the multiset of (row, col, value) is preserved
    a = np.lexsort((v, c, r))
    b = np.lexsort((vout, crd, rows))
    assert np.array_equal(r[a], rows[b]) and np.array_equal(c[a], crd[b]) and np.array_equal(v[a], vout[b])


@pytest.mark.parametrize("order", [0, 1])
def test_power_law_scaled_config4(order):
    c4 = wl.config4(N=50_000, nnz_target=700_000, max_row=30_000)
    coo = c4["coo"]
    _check(50_000, 50_000, coo.levels[0].crd, coo.levels[1].crd, coo.vals, order, what="c4 scaled")


# ---- sizes, input orders and duplicate patterns that stress any sort implementation ----

@pytest.mark.parametrize("nnz", [6143, 6144, 6145, 20_000, 524_288, 524_289, 1_300_000])
def test_sizes_from_thousands_to_a_million(nnz):
    N, M = 90_000, 70_000
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=300 + nnz % 97, dtype=np.float64, sort=False)
    _check(N, M, r, c, v, 0, what=f"nnz={nnz}")


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("kind", ["sorted", "reversed", "by_column", "interleaved"])
def test_unordered_flagged_input_in_special_orders(kind, order):
    """Input flagged unordered that is in fact sorted, reversed, column-major, or a regular
    interleaving of 170 sorted runs."""
    N, M, nnz = 3000, 5000, 700_000
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=41, dtype=np.float32, sort=True)
    if kind == "reversed":
        r, c, v = r[::-1].copy(), c[::-1].copy(), v[::-1].copy()
    elif kind == "by_column":
        o = np.lexsort((r, c))
        r, c, v = r[o], c[o], v[o]
    elif kind == "interleaved":
        stride = len(v) // 4096
        o = np.concatenate([np.arange(len(v))[i::stride] for i in range(stride)])
        r, c, v = r[o], c[o], v[o]
    _check(N, M, r, c, v, order, what=kind)


@pytest.mark.parametrize("order", [0, 1])
def test_many_copies_of_one_coordinate_keep_their_input_order(order):
    """20 000 entries share one (row, col) pair and 9 000 another, scattered through the input."""
    N, M = 4000, 4000
    r, c, v = wl.random_coo_entries(N, M, 300_000, seed=43, dtype=np.float64, sort=False)
    rng = np.random.default_rng(44)
    r = np.concatenate([r, np.full(20_000, 1234), np.full(9_000, 77)])
    c = np.concatenate([c, np.full(20_000, 999), np.full(9_000, 3)])
    p = rng.permutation(len(r))
    r, c = r[p], c[p]
    v = np.arange(len(r), dtype=np.float64)            # values identify the input position
    _check(N, M, r, c, v, order, what="heavy duplicates")
    keep = slice(0, 200_000)
    _check(N, M, r[keep], c[keep], v[keep].astype(np.float32), order, what="heavy duplicates, fp32")


@pytest.mark.parametrize("order", [0, 1])
def test_one_row_holds_most_entries_and_columns_use_31_bits(order):
    rng = np.random.default_rng(45)
    M = 2**31 - 10
    n = 900_000
    r = rng.integers(0, 5000, n)
    r[: 2 * n // 3] = 4321                               # one row with 600 000 entries
    c = rng.integers(0, M, n)
    p = rng.permutation(n)
    _check(5000, M, r[p], c[p], rng.uniform(-1, 1, n), order, what="heavy row, 31-bit columns")
