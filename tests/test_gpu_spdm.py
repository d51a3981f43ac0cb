"""GPU parity: spt_spdm (COO matrix times dense matrix) vs the oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_spdm

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("J", [1, 8, 32, 33, 64, 100])
def test_spdm_ranks(dtype, J):
    N, M = 700, 900
    r, c, v = wl.random_coo_entries(N, M, 30_000, seed=500 + J, dtype=dtype)
    Cm = np.random.default_rng(J).uniform(-1, 1, (M, J)).astype(dtype)
    spec = wl.coo_spec(N, M, r, c, v)
    ref, mag = oracle.spdm(spec, Cm)
    assert_close(gpu_spdm(spec, Cm), ref, mag, dtype, f"spdm J={J}")


@pytest.mark.parametrize("nnz", [0, 1, 1023, 1024, 1025, 300_000])
def test_spdm_sizes_and_power_law_rows(nnz):
    N, M = 5000, 4000
    r, c, v = wl.random_coo_entries(N, M, nnz, seed=600 + nnz, dtype=np.float32, duplicates=True)
    if nnz > 1000:                                  # one heavy row spanning many chunks
        r[: nnz // 2] = 17
        r.sort()
    Cm = np.random.default_rng(1).uniform(-1, 1, (M, 32)).astype(np.float32)
    spec = wl.coo_spec(N, M, r, c, v)
    ref, mag = oracle.spdm(spec, Cm)
    a = gpu_spdm(spec, Cm)
    assert_close(a, ref, mag, np.float32, f"spdm nnz={nnz}")
    assert np.array_equal(a, gpu_spdm(spec, Cm)), "not bit-reproducible"


def test_spdm_exact_integers_and_errors():
    import paper_1804_10112_amd as spt
    import torch
    N, M = 300, 200
    r, c, v = wl.random_coo_entries(N, M, 20_000, seed=3, dtype=np.float32, dist="int", duplicates=True)
    Cm = np.random.default_rng(2).integers(-3, 4, (M, 16)).astype(np.float32)
    spec = wl.coo_spec(N, M, r, c, v)
    ref, _ = oracle.spdm(spec, Cm)
    assert np.array_equal(gpu_spdm(spec, Cm).astype(np.float64), ref)
    B = spt.DeviceTensor(wl.csr_from_sorted_coo(N, M, r, c, v))
    A = torch.zeros(N, 16, device="cuda")
    with pytest.raises(spt.SptError) as e:
        spt.spt_spdm(B, torch.from_numpy(Cm).cuda(), 16, A, None)
    assert e.value.status == 2                      # only COO input
