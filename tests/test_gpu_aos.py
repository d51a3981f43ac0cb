"""GPU parity: array-of-structs COO (one interleaved coordinate array, Section 5.2). spt_spmv splits
the pairs and runs the COO kernels; spt_to_coo, spt_mul_dense and spt_add_to_dense read it per
value; the format-specific operations refuse it and point at spt_to_coo."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_coo_to_csr, gpu_spmv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nnz", [0, 1, 700, 50_000, 400_000])
def test_spmv_aos_coo(dtype, nnz):
    N, M = 3000, 2500
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=5000 + nnz, dtype=dtype)
    x = wl.dense_vector(M, 9, dtype)
    ref, mag = oracle.spmv(wl.coo_spec(N, M, r, c, v), x)
    aos = wl.coo_aos_spec((N, M), (r, c), v)
    oref, _ = oracle.spmv(aos, x)
    assert np.array_equal(oref, ref)                          # the oracle reads the interleaved array itself
    got = gpu_spmv(aos, x, repeat=2)
    assert_close(got[0], ref, mag, dtype, f"aos ordered nnz={nnz}")
    assert np.array_equal(got[0], got[1])                     # ordered: segmented sums
    assert_close(gpu_spmv(aos, x, misalign=True), ref, mag, dtype, "aos misaligned")
    perm = np.random.default_rng(nnz).permutation(len(v))
    shuffled = wl.coo_aos_spec((N, M), (r[perm], c[perm]), v[perm], ordered=False)
    assert_close(gpu_spmv(shuffled, x), ref, mag, dtype, f"aos unordered nnz={nnz}")


def _gpu_to_coo(spec):
    import torch
    import paper_1804_10112_amd as spt
    T = spt.DeviceTensor(spec)
    n = max(len(spec.vals), 1)
    order = len(spec.dims)
    crd = [torch.full((n,), -7, dtype=torch.int32, device="cuda") for _ in range(3)]
    vals = torch.zeros(n, dtype=T.torch_dtype, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    spt.spt_to_coo(T, crd[0], crd[1] if order > 1 else None, crd[2] if order > 2 else None, vals, cnt,
                   T.workspace(spt.SPT_OP_TO_COO))
    torch.cuda.synchronize()
    k = int(cnt.item())
    return [t.cpu().numpy()[:k] for t in crd[:order]], vals.cpu().numpy()[:k]


def test_aos_to_soa_and_on_to_csr():
    N, M = 900, 1100
    r, c, v = wl.random_coo_entries(N, M, 30_000, seed=5100, dtype=np.float64, sort=False)
    aos = wl.coo_aos_spec((N, M), (r, c), v, ordered=False)
    (gr, gc), gv = _gpu_to_coo(aos)
    assert np.array_equal(gr, r) and np.array_equal(gc, c) and np.array_equal(gv, v)
    pos, crd, vals = gpu_coo_to_csr(wl.coo_spec(N, M, gr, gc, gv, ordered=False), 0)
    rpos, rcrd, rvals, _ = oracle.coo_to_csr(N, r, c, v, 0)
    assert np.array_equal(pos, rpos) and np.array_equal(crd, rcrd) and np.array_equal(vals, rvals)
    dims = (30, 40, 50)
    ci, cj, ck, w = wl.random_coo3_entries(dims, 20_000, 5101, dtype=np.float32)
    (gi, gj, gk), gw = _gpu_to_coo(wl.coo_aos_spec(dims, (ci, cj, ck), w))
    assert np.array_equal(gi, ci) and np.array_equal(gj, cj) and np.array_equal(gk, ck) and np.array_equal(gw, w)


def test_aos_elementwise_and_refusals():
    import torch
    import paper_1804_10112_amd as spt
    from test_gpu_elementwise import gpu_add_to_dense, gpu_mul_dense
    N, M = 200, 300
    r, c, v = wl.random_coo_entries(N, M, 5000, seed=5200, dtype=np.float64)
    r2, c2, v2 = wl.random_coo_entries(N, M, 4000, seed=5201, dtype=np.float64)
    aos = wl.coo_aos_spec((N, M), (r, c), v)
    D = np.random.default_rng(1).uniform(-1, 1, (N, M))
    ref = oracle.mul_dense(aos, D)
    assert_close(gpu_mul_dense(aos, D), ref, np.abs(ref), np.float64, "mul_dense aos")
    A, mag = oracle.add_to_dense(aos, wl.csr_from_sorted_coo(N, M, r2, c2, v2))
    got = gpu_add_to_dense(aos, wl.csr_from_sorted_coo(N, M, r2, c2, v2))
    assert_close(got.ravel(), A.ravel(), mag.ravel(), np.float64, "add_to_dense aos + csr")
    T = spt.DeviceTensor(aos)
    i = torch.zeros(6000, dtype=torch.int32, device="cuda")
    w = torch.zeros(6000, dtype=torch.float64, device="cuda")
    with pytest.raises(spt.SptError) as e:
        spt.spt_coo_to_csr(T, 0, i, i, w, torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 2 and "spt_to_coo" in str(e.value)
    with pytest.raises(spt.SptError):
        spt.spt_spmv(T, w, w, None)                              # needs its workspace
