"""GPU parity: spt_innerprod (alpha = sum B_ijk C_ijk on two ordered COO tensors) vs the oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_innerprod

pytestmark = pytest.mark.gpu


def _pair(dims, nb, nc, seed, dtype, skew=None):
    bi, bj, bk, bv = wl.random_coo3_entries(dims, nb, seed, dtype=dtype, dist="u11", skew=skew)
    ci, cj, ck, cv = wl.random_coo3_entries(dims, nc, seed + 1, dtype=dtype, dist="u11")
    return wl.coo3_spec(dims, bi, bj, bk, bv), wl.coo3_spec(dims, ci, cj, ck, cv)


def _check(b, c, dtype, what):
    ref, mag = oracle.innerprod(b, c)
    got = gpu_innerprod(b, c)
    assert_close(got, ref, mag, dtype, what)
    assert got == gpu_innerprod(b, c), f"{what}: not bit-reproducible"
    return ref, mag


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nb,nc", [(1, 1), (50, 70), (2047, 2049), (2048, 5000), (2049, 100),
                                   (20_000, 30_000), (30_000, 9_000)])
def test_innerprod_overlapping_supports(dtype, nb, nc):
    # 60k cells: supports of this density share a good part of their coordinates
    b, c = _pair((40, 30, 50), nb, nc, seed=700 + nb, dtype=dtype)
    ref, mag = _check(b, c, dtype, f"innerprod {nb}x{nc}")
    if min(nb, nc) >= 9000:
        assert mag > 0


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_innerprod_wide_windows_and_skew(dtype):
    # C holds ~90 entries per entry of B: every chunk's window exceeds the LDS window.
    b, c = _pair((64, 64, 128), 5_000, 450_000, seed=11, dtype=dtype, skew=1.2)
    _check(b, c, dtype, "innerprod wide window")
    # and the other way round: windows of a few entries, many chunks
    _check(c, b, dtype, "innerprod narrow window")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_innerprod_dimensions_beyond_63_bits(dtype):
    """Declared dimensions too large for one packed 64-bit key select the three-coordinate
    compare; the stored coordinates (and so the result) are those of the small tensor."""
    dims = (40, 30, 50)
    bi, bj, bk, bv = wl.random_coo3_entries(dims, 20_000, 41, dtype=dtype, dist="u11", skew=1.3)
    ci, cj, ck, cv = wl.random_coo3_entries(dims, 25_000, 42, dtype=dtype, dist="u11")
    ref, mag = oracle.innerprod(wl.coo3_spec(dims, bi, bj, bk, bv), wl.coo3_spec(dims, ci, cj, ck, cv))
    big = (2**31 - 1, 2**30, 2**30)
    got = gpu_innerprod(wl.coo3_spec(big, bi, bj, bk, bv), wl.coo3_spec(big, ci, cj, ck, cv))
    assert mag > 0
    assert_close(got, ref, mag, dtype, "innerprod three-coordinate keys")


def test_innerprod_special_operands():
    dims = (30, 20, 25)
    b, c = _pair(dims, 6000, 6000, seed=21, dtype=np.float64)
    sq = gpu_innerprod(b, b)                                    # <B,B> = sum v^2
    want = float((b.vals.astype(np.float64) ** 2).sum())
    assert abs(sq - want) <= 1e-12 * want
    e = np.zeros(0, np.int32)
    empty = wl.coo3_spec(dims, e, e, e, np.zeros(0, np.float64))
    assert gpu_innerprod(b, empty) == 0.0
    assert gpu_innerprod(empty, b) == 0.0
    assert gpu_innerprod(empty, empty) == 0.0
    # disjoint supports: B in the even k, C in the odd k
    bi, bj, bk, bv = wl.random_coo3_entries((30, 20, 12), 3000, 5, dtype=np.float64)
    ci, cj, ck, cv = wl.random_coo3_entries((30, 20, 12), 3000, 6, dtype=np.float64)
    d1 = wl.coo3_spec(dims, bi, bj, 2 * bk, bv)
    d2 = wl.coo3_spec(dims, ci, cj, 2 * ck + 1, cv)
    assert gpu_innerprod(d1, d2) == 0.0
    # exact small integers
    bi, bj, bk, bv = wl.random_coo3_entries(dims, 9000, 7, dtype=np.float32, dist="int")
    ci, cj, ck, cv = wl.random_coo3_entries(dims, 9000, 8, dtype=np.float32, dist="int")
    b, c = wl.coo3_spec(dims, bi, bj, bk, bv), wl.coo3_spec(dims, ci, cj, ck, cv)
    assert gpu_innerprod(b, c) == oracle.innerprod(b, c)[0]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_innerprod_matrices(dtype):
    N, M = 300, 257
    r1, c1, v1 = wl.random_coo_entries(N, M, 30_000, seed=31, dtype=dtype)
    r2, c2, v2 = wl.random_coo_entries(N, M, 41_000, seed=32, dtype=dtype)
    b, c = wl.coo_spec(N, M, r1, c1, v1), wl.coo_spec(N, M, r2, c2, v2)
    _check(b, c, dtype, "innerprod matrices")


def test_innerprod_full_size_closed_forms():
    """Configuration 5 (50M entries): <B,B> = sum v^2, and <B,C> for C = every third entry of B
    with fresh values plus entries outside B's support = sum over the shared entries."""
    cfg = wl.config5()
    b = cfg["coo"]
    i, j, k = (np.asarray(L.crd) for L in b.levels)
    v = b.vals.astype(np.float64)
    want = float((v * v).sum())
    got = gpu_innerprod(b, b)
    assert abs(got - want) <= 1e-5 * want
    keep = np.arange(0, len(v), 3)
    rng = np.random.default_rng(55)
    w = rng.uniform(-1, 1, keep.size).astype(b.vals.dtype)
    c = wl.coo3_spec(b.dims, i[keep], j[keep], k[keep], w)
    want = float((v[keep] * w.astype(np.float64)).sum())
    mag = float(np.abs(v[keep] * w.astype(np.float64)).sum())
    for got in (gpu_innerprod(b, c), gpu_innerprod(c, b)):
        assert abs(got - want) <= 1e-5 * mag


def test_innerprod_errors():
    import torch
    import paper_1804_10112_amd as spt
    b, c = _pair((10, 10, 10), 100, 100, seed=1, dtype=np.float32)
    B, Ct = spt.DeviceTensor(b), spt.DeviceTensor(c)
    out = torch.zeros(1, device="cuda")
    ws = B.workspace(spt.SPT_OP_INNERPROD)
    with pytest.raises(spt.SptError):
        spt.spt_innerprod(B, Ct, None, ws)
    other = spt.DeviceTensor(_pair((10, 10, 11), 100, 100, seed=1, dtype=np.float32)[1])
    with pytest.raises(spt.SptError) as e:
        spt.spt_innerprod(B, other, out, ws)
    assert "dimension" in str(e.value)
    f64 = spt.DeviceTensor(_pair((10, 10, 10), 100, 100, seed=1, dtype=np.float64)[1])
    with pytest.raises(spt.SptError):
        spt.spt_innerprod(B, f64, out, ws)
    i, j, k, v = wl.random_coo3_entries((10, 10, 10), 100, 3, dtype=np.float32)
    csf = spt.DeviceTensor(wl.csf3_from_sorted_coo((10, 10, 10), i, j, k, v))
    with pytest.raises(spt.SptError):
        spt.spt_innerprod(B, csf, out, ws)
