"""GPU parity: spt_mul_dense (B .* D on B's structure) and spt_add_to_dense (dense A = B + C) on
matrices in every composition, vs the oracle's level walk. Each result value is one rounded
product, or a sum of at most two terms, so results are compared for equality up to the
tolerance of one rounding."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close

pytestmark = pytest.mark.gpu


def _formats(N, M, r, c, v, dense=False):
    out = {
        "coo": wl.coo_spec(N, M, r, c, v),
        "csr": wl.csr_from_sorted_coo(N, M, r, c, v),
        "dcsr": wl.dcsr_from_sorted_coo(N, M, r, c, v),
        "csc": wl.csc_from_coo(N, M, r, c, v),
        "dhash": wl.hashed_rows_from_coo(N, M, r, c, v, W=1 << int(np.ceil(np.log2(2 * max(np.bincount(r).max(), 1) + 1)))),
        "sdia": wl.sparse_dia_from_coo(N, M, r, c, v),
    }
    return out


def gpu_mul_dense(spec, D, ld=None, misalign=False):
    import torch
    import paper_1804_10112_amd as spt
    B = spt.DeviceTensor(spec, misalign=misalign)
    ld = ld or D.shape[1]
    buf = np.full((D.shape[0], ld), np.nan, D.dtype)
    buf[:, :D.shape[1]] = D
    Dd = torch.from_numpy(buf).cuda()
    out = torch.full((max(len(spec.vals), 1),), float("nan"), dtype=B.torch_dtype, device="cuda")
    spt.spt_mul_dense(B, Dd, ld, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()[:len(spec.vals)]


def gpu_add_to_dense(bspec, cspec, ld=None):
    import torch
    import paper_1804_10112_amd as spt
    B, Ct = spt.DeviceTensor(bspec), spt.DeviceTensor(cspec)
    N, M = bspec.dims
    ld = ld or M
    A = torch.full((N, ld), float("nan"), dtype=B.torch_dtype, device="cuda")
    spt.spt_add_to_dense(B, Ct, A, ld)
    torch.cuda.synchronize()
    return A.cpu().numpy()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nnz", [1, 500, 30_000])
def test_mul_dense_every_composition(dtype, nnz):
    N, M = 300, 421
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=4000 + nnz, dtype=dtype)
    D = np.random.default_rng(nnz).uniform(-1, 1, (N, M)).astype(dtype)
    for name, spec in _formats(N, M, r, c, v).items():
        ref = oracle.mul_dense(spec, D)
        got = gpu_mul_dense(spec, D, ld=M + (5 if name == "csr" else 0), misalign=name == "coo")
        assert_close(got, ref, np.abs(ref), dtype, f"mul_dense {name} nnz={nnz}")
    c3 = wl.config3(N=500, lo=0, hi=12, seed=41, dtype=dtype)   # ELL: padding positions give 0
    D3 = np.random.default_rng(42).uniform(-1, 1, c3["ell"].dims).astype(dtype)
    ref = oracle.mul_dense(c3["ell"], D3)
    got = gpu_mul_dense(c3["ell"], D3)
    assert_close(got, ref, np.abs(ref), dtype, "mul_dense ell")
    assert not got[c3["ell"].levels[2].crd < 0].any()
    c2 = wl.config2(N=400, dtype=dtype, poison=True)            # DIA: cells outside the matrix give 0
    D2 = np.random.default_rng(43).uniform(-1, 1, c2["dia"].dims).astype(dtype)
    ref = oracle.mul_dense(c2["dia"], D2)
    got = gpu_mul_dense(c2["dia"], D2)
    assert not np.isnan(got).any()
    assert_close(got, ref, np.abs(ref), dtype, "mul_dense dia")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_add_to_dense_mixed_formats(dtype):
    N, M = 211, 307
    r1, c1, v1 = wl.random_coo_entries(N, M, 9000, seed=4100, dtype=dtype)
    r2, c2, v2 = wl.random_coo_entries(N, M, 12000, seed=4101, dtype=dtype)
    fb, fc = _formats(N, M, r1, c1, v1), _formats(N, M, r2, c2, v2)
    ref, mag = oracle.add_to_dense(fb["csr"], fc["coo"])
    for nb, nc in (("csr", "coo"), ("coo", "csc"), ("dcsr", "dhash"), ("sdia", "csr"), ("csc", "csc")):
        got = gpu_add_to_dense(fb[nb], fc[nc])
        assert_close(got.ravel(), ref.ravel(), mag.ravel(), dtype, f"add_to_dense {nb}+{nc}")
    padded = gpu_add_to_dense(fb["csr"], fc["coo"], ld=M + 3)
    assert_close(padded[:, :M].ravel(), ref.ravel(), mag.ravel(), dtype, "add_to_dense ld")
    assert np.isnan(padded[:, M:]).all()                        # cells beyond M are not touched
    e = np.zeros(0, np.int32)
    empty = wl.coo_spec(N, M, e, e, np.zeros(0, dtype))
    assert not gpu_add_to_dense(empty, empty).any()
    only_b = gpu_add_to_dense(fb["coo"], empty)
    want = np.zeros((N, M), dtype)
    want[r1, c1] = v1
    assert np.array_equal(only_b, want)


def test_elementwise_errors():
    import torch
    import paper_1804_10112_amd as spt
    r, c, v = wl.random_coo_entries(20, 30, 50, seed=1, dtype=np.float32)
    B = spt.DeviceTensor(wl.coo_spec(20, 30, r, c, v))
    D = torch.zeros(20, 30, device="cuda")
    out = torch.zeros(50, device="cuda")
    with pytest.raises(spt.SptError):
        spt.spt_mul_dense(B, D, 29, out)                         # ld below the column count
    with pytest.raises(spt.SptError):
        spt.spt_mul_dense(B, None, 30, out)
    other = spt.DeviceTensor(wl.coo_spec(20, 31, r, c, v))
    A = torch.zeros(20, 31, device="cuda")
    with pytest.raises(spt.SptError):
        spt.spt_add_to_dense(B, other, A, 31)                    # shapes differ
    ci, cj, ck, w = wl.random_coo3_entries((5, 5, 5), 20, 2, dtype=np.float32)
    t3 = spt.DeviceTensor(wl.coo3_spec((5, 5, 5), ci, cj, ck, w))
    with pytest.raises(spt.SptError):
        spt.spt_mul_dense(t3, D, 30, out)                        # no matrix
