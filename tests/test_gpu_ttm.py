"""GPU parity: spt_ttm (A_ijk = sum_l B_ijl C_kl on ordered COO and on CSF) vs the oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_ttm

pytestmark = pytest.mark.gpu


def _case(dims, nnz, K, seed, dtype, skew=1.5):
    ci, cj, cl, v = wl.random_coo3_entries(dims, nnz, seed, dtype=dtype, dist="u11", skew=skew)
    Cm = np.random.default_rng(seed + 9).uniform(-1, 1, (K, dims[2])).astype(dtype)
    return (wl.coo3_spec(dims, ci, cj, cl, v), wl.csf3_from_sorted_coo(dims, ci, cj, cl, v), Cm)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("K", [1, 8, 32, 33, 64, 100])
def test_ttm_ranks(dtype, K):
    coo, csf, Cm = _case((60, 50, 70), 40_000, K, seed=800 + K, dtype=dtype)
    ri, rj, rv, rm = oracle.ttm(coo, Cm)
    gi, gj, gv = gpu_ttm(coo, Cm)
    assert np.array_equal(gi, ri) and np.array_equal(gj, rj)
    assert_close(gv, rv, rm, dtype, f"ttm coo K={K}")
    _, _, fv = gpu_ttm(csf, Cm, is_csf=True)
    assert fv.shape == rv.shape
    assert_close(fv, rv, rm, dtype, f"ttm csf K={K}")


@pytest.mark.parametrize("nnz", [1, 2047, 2048, 2049, 4097, 150_000])
def test_ttm_sizes_and_long_fibres(nnz):
    # 12 x 9 fibres only: at 150k entries every fibre spans many chunks of every kernel
    coo, csf, Cm = _case((12, 9, 3000), nnz, 32, seed=900 + nnz, dtype=np.float32, skew=1.2)
    ri, rj, rv, rm = oracle.ttm(coo, Cm)
    gi, gj, gv = gpu_ttm(coo, Cm)
    assert np.array_equal(gi, ri) and np.array_equal(gj, rj)
    assert_close(gv, rv, rm, np.float32, f"ttm coo nnz={nnz}")
    assert_close(gpu_ttm(csf, Cm, is_csf=True)[2], rv, rm, np.float32, f"ttm csf nnz={nnz}")
    assert np.array_equal(gv, gpu_ttm(coo, Cm)[2]), "not bit-reproducible"
    mi, mj, mv = gpu_ttm(coo, Cm, misalign=True)            # arrays off 16-byte alignment: scalar loads
    assert np.array_equal(mi, ri) and np.array_equal(mj, rj) and np.array_equal(mv, gv)


def test_ttm_singleton_fibres_and_exact_integers():
    # very sparse: almost every fibre holds one entry (the shape of configuration 5)
    dims = (3000, 2500, 400)
    ci, cj, cl, v = wl.random_coo3_entries(dims, 60_000, 77, dtype=np.float32, dist="int")
    Cm = np.random.default_rng(3).integers(-3, 4, (16, dims[2])).astype(np.float32)
    coo = wl.coo3_spec(dims, ci, cj, cl, v)
    ri, rj, rv, _ = oracle.ttm(coo, Cm)
    gi, gj, gv = gpu_ttm(coo, Cm)
    assert len(ri) > 59_000
    assert np.array_equal(gi, ri) and np.array_equal(gj, rj)
    assert np.array_equal(gv.astype(np.float64), rv)
    csf = wl.csf3_from_sorted_coo(dims, ci, cj, cl, v)
    assert np.array_equal(gpu_ttm(csf, Cm, is_csf=True)[2].astype(np.float64), rv)


def test_ttm_empty_and_errors():
    import torch
    import paper_1804_10112_amd as spt
    e = np.zeros(0, np.int32)
    empty = wl.coo3_spec((4, 4, 4), e, e, e, np.zeros(0, np.float32))
    gi, gj, gv = gpu_ttm(empty, np.ones((3, 4), np.float32))
    assert len(gi) == 0 and gv.shape == (0, 3)
    coo, _, Cm = _case((10, 10, 10), 200, 4, seed=1, dtype=np.float32)
    B = spt.DeviceTensor(coo)
    Cd = torch.from_numpy(Cm).cuda()
    ov = torch.zeros(200, 4, device="cuda")
    oi = torch.zeros(200, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    ws = B.workspace(spt.SPT_OP_TTM, 4)
    with pytest.raises(spt.SptError):
        spt.spt_ttm(B, Cd, 0, oi, oi, ov, cnt, ws)
    with pytest.raises(spt.SptError):
        spt.spt_ttm(B, Cd, 4, oi, oi, ov, None, ws)             # COO output needs the count
    with pytest.raises(spt.SptError) as err:
        spt.spt_ttm(B, Cd, 4, oi, oi, ov, cnt, None)
    assert "workspace" in str(err.value)
    r, c, v = wl.random_coo_entries(10, 10, 30, seed=2, dtype=np.float32)
    with pytest.raises(spt.SptError):
        spt.spt_ttm(spt.DeviceTensor(wl.coo_spec(10, 10, r, c, v)), Cd, 4, oi, oi, ov, cnt, ws)


def test_ttm_full_size_sampled():
    """Configuration 5 at full size with K = 8: fibre coordinates against numpy's unique, the
    CSF output bit-equal in shape, and sampled fibres against the oracle run on exactly those
    fibres' entries."""
    cfg = wl.config5()
    coo, csf = cfg["coo"], cfg["csf"]
    K = 8
    Cm = np.random.default_rng(81).uniform(0, 1, (K, coo.dims[2])).astype(np.float32)
    i, j, l = (np.asarray(L.crd) for L in coo.levels)
    key = i.astype(np.int64) * coo.dims[1] + j
    head = np.concatenate([[True], key[1:] != key[:-1]])
    gi, gj, gv = gpu_ttm(coo, Cm)
    assert len(gi) == int(head.sum())
    assert np.array_equal(gi, i[head]) and np.array_equal(gj, j[head])
    _, _, fv = gpu_ttm(csf, Cm, is_csf=True)
    assert fv.shape == gv.shape
    fid = np.cumsum(head) - 1
    rng = np.random.default_rng(5)
    counts = np.bincount(fid)
    sample = np.unique(np.concatenate([rng.integers(0, len(gi), 300), np.argsort(counts)[-3:],
                                       [0, len(gi) - 1]]))
    pick = np.isin(fid, sample)
    sub = wl.coo3_spec(coo.dims, i[pick], j[pick], l[pick], coo.vals[pick])
    ri, rj, rv, rm = oracle.ttm(sub, Cm)
    assert np.array_equal(ri, gi[sample]) and np.array_equal(rj, gj[sample])
    assert_close(gv[sample], rv, rm, np.float32, "ttm coo full size sample")
    assert_close(fv[sample], rv, rm, np.float32, "ttm csf full size sample")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_ttm_csf_with_empty_fibres(dtype):
    """A fibre position without entries still owns K output values: they must come back 0, not
    whatever the (NaN-prefilled) buffer held."""
    dims = (700, 50, 90)
    ci, cj, cl, v = wl.random_coo3_entries(dims, 8000, 31, dtype=dtype, dist="u11", skew=1.5)
    gap = wl.csf3_with_empty_segments(dims, ci, cj, cl, v, seed=32, extra_fibers=5000, extra_slices=50)
    p2 = np.asarray(gap.levels[2].pos)
    full = np.diff(p2) > 0
    for K in (5, 32):
        Cm = np.random.default_rng(K).uniform(-1, 1, (K, dims[2])).astype(dtype)
        ri, rj, rv, rm = oracle.ttm(wl.coo3_spec(dims, ci, cj, cl, v), Cm)
        _, _, fv = gpu_ttm(gap, Cm, is_csf=True, fiber_capacity=len(full))
        assert fv.shape == (len(full), K)
        assert np.all(fv[~full] == 0), "values of empty fibres"
        assert_close(fv[full], rv, rm, dtype, f"ttm csf with gaps K={K}")
