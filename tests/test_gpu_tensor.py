"""GPU parity: spt_ttv and spt_mttkrp (COO and CSF) vs the oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_mttkrp, gpu_ttv

pytestmark = pytest.mark.gpu


def _tensor(dims, nnz, seed, dtype, skew=1.5, dist="u01"):
    ci, cj, ck, v = wl.random_coo3_entries(dims, nnz, seed, dtype, dist, skew=skew)
    return (wl.coo3_spec(dims, ci, cj, ck, v), wl.csf3_from_sorted_coo(dims, ci, cj, ck, v))


def _check_ttv(coo, csf, c, what):
    ri, rj, rv, rm = oracle.ttv(coo, c)
    oi, oj, ov, n = gpu_ttv(coo, c)
    assert n == len(ri), f"{what}: fiber count {n} != {len(ri)}"
    assert np.array_equal(oi, ri) and np.array_equal(oj, rj), f"{what}: output coordinates differ"
    assert_close(ov, rv, rm, coo.vals.dtype, what + " coo")
    _, _, cv, n2 = gpu_ttv(csf, c)
    assert n2 == len(ri)
    assert_close(cv, rv, rm, coo.vals.dtype, what + " csf")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nnz", [1, 200, 2047, 2048, 2049, 6000, 150_000])
def test_ttv_random(dtype, nnz):
    dims = (300, 41, 57)
    coo, csf = _tensor(dims, nnz, 300 + nnz, dtype)
    c = wl.dense_vector(dims[2], 1, dtype, "u01")
    _check_ttv(coo, csf, c, f"ttv nnz={nnz}")


def test_ttv_degenerate():
    # one fiber holds everything (spans chunks); single-entry fibers; empty tensor
    n = 5000
    k = np.arange(n)
    v = np.random.default_rng(0).uniform(0, 1, n).astype(np.float32)
    c = wl.dense_vector(n, 2, np.float32, "u01")
    z = np.zeros(n, int)
    _check_ttv(wl.coo3_spec((3, 3, n), z + 2, z + 1, k, v), wl.csf3_from_sorted_coo((3, 3, n), z + 2, z + 1, k, v),
               c, "one fiber")
    _check_ttv(wl.coo3_spec((n, 2, n), k, z, k, v), wl.csf3_from_sorted_coo((n, 2, n), k, z, k, v),
               c, "singleton fibers")
    e = np.zeros(0, int)
    oi, oj, ov, cnt = gpu_ttv(wl.coo3_spec((3, 3, 3), e, e, e, np.zeros(0, np.float32)), c[:3])
    assert cnt == 0
    # a fiber whose sum cancels is still emitted
    coo = wl.coo3_spec((2, 2, 2), [0, 0], [1, 1], [0, 1], np.array([1.0, -1.0]))
    oi, oj, ov, cnt = gpu_ttv(coo, np.ones(2))
    assert cnt == 1 and oi[0] == 0 and oj[0] == 1 and ov[0] == 0.0


def test_ttv_exact_integer_is_bit_exact():
    dims = (50, 60, 70)
    coo, csf = _tensor(dims, 40_000, 7, np.float32, dist="int")
    c = wl.dense_vector(70, 3, np.float32, "int")
    ri, rj, rv, _ = oracle.ttv(coo, c)
    oi, oj, ov, n = gpu_ttv(coo, c)
    assert np.array_equal(ov.astype(np.float64), rv)
    assert np.array_equal(gpu_ttv(csf, c)[2].astype(np.float64), rv)


def _check_mttkrp(coo, csf, Cm, Dm, what):
    ref, mag = oracle.mttkrp(coo, Cm, Dm)
    assert_close(gpu_mttkrp(coo, Cm, Dm), ref, mag, coo.vals.dtype, what + " coo")
    assert_close(gpu_mttkrp(csf, Cm, Dm), ref, mag, coo.vals.dtype, what + " csf")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("J", [1, 8, 16, 24, 32, 33, 64, 100, 128, 260])
def test_mttkrp_ranks(dtype, J):
    dims = (200, 37, 53)
    coo, csf = _tensor(dims, 20_000, 400 + J, dtype)
    rng = np.random.default_rng(J)
    Cm = rng.uniform(0, 1, (dims[1], J)).astype(dtype)
    Dm = rng.uniform(0, 1, (dims[2], J)).astype(dtype)
    _check_mttkrp(coo, csf, Cm, Dm, f"mttkrp J={J}")


@pytest.mark.parametrize("nnz", [1, 127, 128, 129, 1023, 1024, 1025, 5000, 300_000])
def test_mttkrp_sizes(nnz):
    dims = (500, 64, 81)
    coo, csf = _tensor(dims, nnz, 500 + nnz, np.float32)
    rng = np.random.default_rng(nnz)
    Cm = rng.uniform(0, 1, (dims[1], 32)).astype(np.float32)
    Dm = rng.uniform(0, 1, (dims[2], 32)).astype(np.float32)
    _check_mttkrp(coo, csf, Cm, Dm, f"mttkrp nnz={nnz}")


def test_mttkrp_degenerate_and_exact():
    rng = np.random.default_rng(1)
    # one slice holds everything (crosses many chunks and both carry levels)
    n = 200_000
    k = rng.integers(0, 300, n)
    l = rng.integers(0, 400, n)
    key = np.unique(k * 400 + l)
    k, l = key // 400, key % 400
    v = rng.integers(-3, 4, len(key)).astype(np.float32)
    Cm = rng.integers(-3, 4, (300, 32)).astype(np.float32)
    Dm = rng.integers(-3, 4, (400, 32)).astype(np.float32)
    for row in (0, 4):
        i = np.full(len(key), row)
        coo = wl.coo3_spec((5, 300, 400), i, k, l, v)
        csf = wl.csf3_from_sorted_coo((5, 300, 400), i, k, l, v)
        ref, _ = oracle.mttkrp(coo, Cm, Dm)
        assert np.array_equal(gpu_mttkrp(coo, Cm, Dm).astype(np.float64), ref), "coo one slice"
        assert np.array_equal(gpu_mttkrp(csf, Cm, Dm).astype(np.float64), ref), "csf one slice"
    # empty tensor: A is all zeros
    e = np.zeros(0, int)
    A = gpu_mttkrp(wl.coo3_spec((5, 300, 400), e, e, e, np.zeros(0, np.float32)), Cm, Dm)
    assert np.array_equal(A, np.zeros((5, 32), np.float32))


def test_buffers_that_are_not_16_byte_aligned():
    dims = (300, 41, 57)
    coo, csf = _tensor(dims, 9000, 11, np.float32)
    c = wl.dense_vector(dims[2], 1, np.float32, "u01")
    ri, rj, rv, rm = oracle.ttv(coo, c)
    oi, oj, ov, n = gpu_ttv(coo, c, misalign=True)
    assert n == len(ri) and np.array_equal(oi, ri) and np.array_equal(oj, rj)
    assert_close(ov, rv, rm, np.float32, "ttv coo misaligned")
    assert_close(gpu_ttv(csf, c, misalign=True)[2], rv, rm, np.float32, "ttv csf misaligned")
    rng = np.random.default_rng(3)
    Cm = rng.uniform(0, 1, (dims[1], 32)).astype(np.float32)
    Dm = rng.uniform(0, 1, (dims[2], 32)).astype(np.float32)
    ref, mag = oracle.mttkrp(coo, Cm, Dm)
    assert_close(gpu_mttkrp(coo, Cm, Dm, misalign=True), ref, mag, np.float32, "mttkrp coo misaligned")
    assert_close(gpu_mttkrp(csf, Cm, Dm, misalign=True), ref, mag, np.float32, "mttkrp csf misaligned")


def test_scaled_config5():
    c5 = wl.config5(dims=(2000, 1600, 1000), nnz=400_000)
    _check_ttv(c5["coo"], c5["csf"], c5["c"], "c5 ttv")
    _check_mttkrp(c5["coo"], c5["csf"], c5["C"], c5["D"], "c5 mttkrp")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nnz,extra", [(300, 400), (5000, 3000), (60_000, 20_000)])
def test_csf_with_empty_fibres_and_slices(dtype, nnz, extra):
    """Empty segments in the compressed levels (first, middle and last fibre of a slice empty,
    slices made of empty fibres only, slices without fibres) against the unfactored oracle."""
    dims = (20_000, 60, 70)
    ci, ck, cl, v = wl.random_coo3_entries(dims, nnz, 700 + nnz, dtype, "u01", skew=1.5)
    coo = wl.coo3_spec(dims, ci, ck, cl, v)
    gap = wl.csf3_with_empty_segments(dims, ci, ck, cl, v, seed=nnz, extra_fibers=extra, extra_slices=200)
    p1, p2 = np.asarray(gap.levels[1].pos), np.asarray(gap.levels[2].pos)
    lead = p1[:-1][np.diff(p1) > 0]
    assert (np.diff(p2)[lead] == 0).sum() > 0 and (np.diff(p1) == 0).sum() > 0
    rng = np.random.default_rng(nnz)
    for J in (32, 40):
        Cm = rng.uniform(0, 1, (dims[1], J)).astype(dtype)
        Dm = rng.uniform(0, 1, (dims[2], J)).astype(dtype)
        ref, mag = oracle.mttkrp(coo, Cm, Dm)
        assert_close(gpu_mttkrp(gap, Cm, Dm), ref, mag, dtype, f"mttkrp csf with gaps J={J}")
    # TTV: one value per fibre position, 0 for a fibre without entries
    c = wl.dense_vector(dims[2], 5, dtype, "u01")
    ri, rj, rv, rm = oracle.ttv(coo, c)
    _, _, ov, n = gpu_ttv(gap, c)
    full = np.diff(p2) > 0
    assert n == len(full) and np.all(ov[~full] == 0)
    assert_close(ov[full], rv, rm, dtype, "ttv csf with gaps")


WAVE_MIN = 1 << 18  # from this many entries on TTV keeps c in LDS and lets every wave walk on its own


@pytest.mark.parametrize("dtype,K", [(np.float32, 900), (np.float32, 32_768), (np.float32, 50_000),
                                     (np.float64, 16_384), (np.float64, 16_385), (np.float64, 40_000)])
@pytest.mark.parametrize("tail", [0, 1, 2, 3])
def test_ttv_with_the_vector_in_lds(dtype, K, tail):
    """Large tensors: c is cached in LDS whole (K up to 128 KiB of values) or in part (the
    rest is gathered from global memory); the entry count takes every remainder modulo 4, so
    the last 16-byte group and the last 256-entry piece of a wave are partial."""
    dims = (3000, 500, K)
    ci, cj, ck, v = wl.random_coo3_entries(dims, WAVE_MIN + 40_000, 900 + K % 97 + tail, dtype, "u01", skew=1.5)
    n = len(v) - (len(v) - tail) % 4
    ci, cj, ck, v = ci[:n], cj[:n], ck[:n], v[:n]
    assert n >= WAVE_MIN and n % 4 == tail
    coo, csf = wl.coo3_spec(dims, ci, cj, ck, v), wl.csf3_from_sorted_coo(dims, ci, cj, ck, v)
    c = wl.dense_vector(K, 7, dtype, "u01")
    _check_ttv(coo, csf, c, f"ttv in LDS K={K} tail={tail}")


def test_large_ttv_with_a_vector_far_beyond_lds_takes_the_chunked_kernels():
    """c of 600 000 values: less than a quarter would fit LDS, the chunked kernels run."""
    dims = (300, 500, 600_000)
    coo, csf = _tensor(dims, WAVE_MIN + 30_000, 77, np.float32)
    assert len(coo.vals) >= WAVE_MIN
    _check_ttv(coo, csf, wl.dense_vector(dims[2], 3, np.float32, "u01"), "ttv, K = 600 000")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_ttv_in_lds_with_long_fibres_empty_fibres_and_unaligned_buffers(dtype):
    """Fibres of 1 to 3000 entries (several 256-entry pieces: chains of carries), a CSF with
    empty fibres and slices, exact small-integer data (bit-exact sums), unaligned arrays."""
    rng = np.random.default_rng(17)
    dims = (400, 300, 4000)
    lens = np.minimum(rng.zipf(1.3, 9000), 3000)
    fib = np.sort(rng.choice(dims[0] * dims[1], len(lens), replace=False))
    ci, cj = np.repeat(fib // dims[1], lens), np.repeat(fib % dims[1], lens)
    ck = np.concatenate([np.sort(rng.choice(dims[2], l, replace=False)) for l in lens])
    v = rng.integers(-3, 4, len(ck)).astype(dtype)
    assert len(v) >= WAVE_MIN, len(v)
    c = rng.integers(-2, 3, dims[2]).astype(dtype)
    coo, csf = wl.coo3_spec(dims, ci, cj, ck, v), wl.csf3_from_sorted_coo(dims, ci, cj, ck, v)
    ri, rj, rv, _ = oracle.ttv(coo, c)
    for misalign in (False, True):
        oi, oj, ov, n = gpu_ttv(coo, c, misalign=misalign)
        assert n == len(ri) and np.array_equal(oi, ri) and np.array_equal(oj, rj)
        assert np.array_equal(ov.astype(np.float64), rv), "coo"
        assert np.array_equal(gpu_ttv(csf, c, misalign=misalign)[2].astype(np.float64), rv), "csf"
    gap = wl.csf3_with_empty_segments(dims, ci, cj, ck, v, seed=3, extra_fibers=30_000, extra_slices=100)
    p2 = np.asarray(gap.levels[2].pos)
    full = np.diff(p2) > 0
    assert (~full).sum() > 1000
    _, _, gv, n = gpu_ttv(gap, c)
    assert n == len(full) and np.all(gv[~full] == 0)
    assert np.array_equal(gv[full].astype(np.float64), rv), "csf with gaps"


def test_mttkrp_with_a_dimension_beyond_24_bits_takes_the_general_addressing():
    """Coordinates from 2^23 on do not fit the 24-bit multiply of the fast factor addressing."""
    dims = (70, 9_000_000, 50)
    rng = np.random.default_rng(8)
    n = 30_000
    key = np.unique(rng.integers(0, 70, n) * (9_000_000 * 50) + rng.integers(8_900_000, 9_000_000, n) * 50
                    + rng.integers(0, 50, n))
    ci, ck, cl = key // (9_000_000 * 50), (key // 50) % 9_000_000, key % 50
    v = rng.uniform(0, 1, len(key)).astype(np.float32)
    coo = wl.coo3_spec(dims, ci, ck, cl, v)
    csf = wl.csf3_from_sorted_coo(dims, ci, ck, cl, v)
    Cm = np.zeros((dims[1], 4), np.float32)
    Cm[8_900_000:] = rng.uniform(0, 1, (100_000, 4)).astype(np.float32)
    Dm = rng.uniform(0, 1, (dims[2], 4)).astype(np.float32)
    _check_mttkrp(coo, csf, Cm, Dm, "mttkrp, 9M-row factor")
