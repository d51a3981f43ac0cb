"""spt_spmv_static (the entry point that allocates nothing: its scratch memory is a fixed
array inside the library) against spt_spmv with a caller workspace, through the C ABI."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _both(spec, x):
    """y of spt_spmv (workspace from torch) and of spt_spmv_static on the same operands."""
    import torch
    import paper_1804_10112_amd as spt
    A = spt.DeviceTensor(spec)
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    y_ws = torch.full((spec.dims[0],), float("nan"), dtype=A.torch_dtype, device="cuda")
    y_st = torch.full((spec.dims[0],), float("nan"), dtype=A.torch_dtype, device="cuda")
    spt.spt_spmv(A, xd, y_ws, A.workspace(spt.SPT_OP_SPMV))
    spt.spt_spmv_static(A, xd, y_st)
    torch.cuda.synchronize()
    return y_ws.cpu().numpy(), y_st.cpu().numpy()


def _power_law(N, nnz, max_row, seed):
    c4 = wl.config4(N=N, nnz_target=nnz, max_row=max_row, seed=seed, with_sorted=True)
    r, c, v = c4["sorted"]
    return c4, wl.csr_from_sorted_coo(N, N, r, c, v), wl.coo_spec(N, N, r, c, v, ordered=True)


@pytest.mark.parametrize("fmt", ["csr", "coo_sorted", "coo_unordered"])
def test_two_calls_in_a_row_second_smaller(fmt):
    import oracle
    from gpu_util import assert_close
    # rows of up to 30 000 entries: the entry-balanced kernel with carries across many chunks
    # (the binned scatter of an unordered COO needs ~12 bytes per entry: 250 000 entries fit)
    sizes = ((60_000, 900_000, 30_000, 11), (5_000, 40_000, 3_000, 12))
    if fmt == "coo_unordered":
        sizes = ((20_000, 250_000, 8_000, 11), (5_000, 40_000, 3_000, 12), (500, 3_000, 100, 13))
    for N, nnz, max_row, seed in sizes:
        c4, csr, coo = _power_law(N, nnz, max_row, seed)
        spec = {"csr": csr, "coo_sorted": coo, "coo_unordered": c4["coo"]}[fmt]
        y_ws, y_st = _both(spec, c4["x"])
        ref, mag = oracle.spmv(spec, c4["x"])
        assert_close(y_st, ref, mag, np.float64, f"static {fmt} N={N}")
        if fmt != "coo_unordered":       # deterministic kernels: the two entry points agree bit for bit
            assert np.array_equal(y_ws, y_st)
        else:
            assert_close(y_ws, ref, mag, np.float64, f"workspace {fmt} N={N}")


def test_formats_without_scratch_and_fp32():
    import oracle
    from gpu_util import assert_close
    c2 = wl.config2(N=30_000)
    c3 = wl.config3(N=30_000)
    for spec, x, dt in ((c2["dia"], c2["x"], np.float64), (c3["ell"], c3["x"], np.float32),
                        (c3["csr"], c3["x"], np.float32)):
        y_ws, y_st = _both(spec, x)
        ref, mag = oracle.spmv(spec, x)
        assert_close(y_st, ref, mag, dt, "static")
        assert np.array_equal(y_ws, y_st)


def test_refuses_what_does_not_fit():
    import torch
    import paper_1804_10112_amd as spt
    N, nnz = 100_000, 1_000_000          # unordered COO: the binned scatter needs ~12 MB
    rng = np.random.default_rng(3)
    spec = wl.coo_spec(N, N, rng.integers(0, N, nnz, dtype=np.int32), rng.integers(0, N, nnz, dtype=np.int32),
                       rng.uniform(-1, 1, nnz), ordered=False)
    A = spt.DeviceTensor(spec)
    assert spt.spt_workspace_bytes(spt.SPT_OP_SPMV, A) > spt.SPT_STATIC_SCRATCH_BYTES
    x = torch.zeros(N, dtype=torch.float64, device="cuda")
    y = torch.full((N,), 7.0, dtype=torch.float64, device="cuda")
    with pytest.raises(spt.SptError) as e:
        spt.spt_spmv_static(A, x, y)
    assert e.value.status == spt.binding.SPT_ERR_WORKSPACE and "static" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)            # nothing was launched
