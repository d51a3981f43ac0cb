"""GPU parity: CSR SpMV with x stored as a sparse vector (compressed level) or
a hash map (hashed level, locate with linear probing) vs the oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_spmv, gpu_spmv_sparse_x

pytestmark = pytest.mark.gpu


def _matrix(dtype, N=3000, M=5000, nnz=60_000, seed=71):
    r, c, v = wl.random_coo_entries(N, M, nnz, seed, dtype)
    return wl.csr_from_sorted_coo(N, M, r, c, v)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("nnzx", [0, 1, 17, 700, 5000])
def test_sparse_vector_x(dtype, nnzx):
    A = _matrix(dtype)
    xc, xv = wl.random_sparse_vector(5000, nnzx, seed=72 + nnzx, dtype=dtype)
    X = wl.sparse_vector_spec(5000, xc, xv)
    ref, mag = oracle.spmv_sparse_x(A, X)
    assert_close(gpu_spmv_sparse_x(A, X), ref, mag, dtype, f"sparse x nnz={nnzx}")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("nnzx,W", [(0, 1), (0, 13), (1, 1), (40, 40), (40, 41), (700, 701),
                                    (700, 1024), (700, 4096), (5000, 5000), (5000, 8191)])
def test_hash_map_x(dtype, nnzx, W):
    A = _matrix(dtype)
    xc, xv = wl.random_sparse_vector(5000, nnzx, seed=90 + nnzx + W, dtype=dtype)
    X = wl.hash_vector_spec(5000, xc, xv, W)
    ref, mag = oracle.spmv_sparse_x(A, X)
    got = gpu_spmv_sparse_x(A, X)
    assert_close(got, ref, mag, dtype, f"hash x nnz={nnzx} W={W}")
    # the three formats of the same x give the same y (Figure 16 compares only their speed)
    xd = np.zeros(5000, dtype)
    xd[xc] = xv
    dense = gpu_spmv(A, xd)
    sparse = gpu_spmv_sparse_x(A, wl.sparse_vector_spec(5000, xc, xv))
    assert np.array_equal(got, dense) and np.array_equal(sparse, dense)


def test_clustered_keys_probe_across_the_wrap():
    """All coordinates collide on the last buckets, so probing wraps to the table start."""
    A = _matrix(np.float64)
    W = 64
    xc = np.array([63, 127, 191, 255, 319, 62, 126], np.int32)    # i % 64 in {63, 62}
    xv = np.arange(1.0, 8.0)
    o = np.argsort(xc)
    X = wl.hash_vector_spec(5000, xc, xv, W)
    ref, mag = oracle.spmv_sparse_x(A, X)
    assert_close(gpu_spmv_sparse_x(A, X), ref, mag, np.float64, "wrapping probes")
    S = wl.sparse_vector_spec(5000, xc[o], xv[o])
    assert_close(gpu_spmv_sparse_x(A, S), ref, mag, np.float64, "same x as sparse vector")


def test_invalid_x_descriptors():
    import paper_1804_10112_amd as spt
    import torch
    A = spt.DeviceTensor(_matrix(np.float64))
    y = torch.zeros(3000, dtype=torch.float64, device="cuda")
    ws = A.workspace(spt.SPT_OP_SPMV)
    xc, xv = wl.random_sparse_vector(5000, 10, seed=1)
    X32 = spt.DeviceTensor(wl.sparse_vector_spec(5000, xc, xv.astype(np.float32)))
    with pytest.raises(spt.SptError) as e:
        spt.spt_spmv_sparse_x(A, X32, y, ws)                 # dtype mismatch
    assert e.value.status == 1
    H = spt.DeviceTensor(wl.hash_vector_spec(5000, xc, xv, 16))
    H.c.level[0].flags |= spt.SPT_ORDERED                    # Table 1: hashed cannot be ordered
    with pytest.raises(spt.SptError) as e:
        spt.spt_spmv_sparse_x(A, H, y, ws)
    assert e.value.status == 1
    coo = spt.DeviceTensor(wl.coo_spec(3000, 5000, [0], [0], np.ones(1)))
    X = spt.DeviceTensor(wl.sparse_vector_spec(5000, xc, xv))
    with pytest.raises(spt.SptError) as e:
        spt.spt_spmv_sparse_x(coo, X, y, ws)                 # A must be CSR
    assert e.value.status == 2
