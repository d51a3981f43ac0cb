"""GPU parity: the packers (COO3 -> CSF, COO/CSR -> ELL, COO -> DIA) vs the oracle: every
output array bit-exact; the packed tensors are then fed back to the kernels that consume them."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close, gpu_mttkrp, gpu_spmv

pytestmark = pytest.mark.gpu


def gpu_to_csf(spec, misalign=False):
    import torch
    import paper_1804_10112_amd as spt
    B = spt.DeviceTensor(spec, misalign=misalign)
    n = max(len(spec.vals), 1)
    i32 = lambda m: torch.full((m,), -7, dtype=torch.int32, device="cuda")
    pos0, crd0, pos1, crd1, pos2, crd2 = i32(2), i32(n), i32(n + 1), i32(n), i32(n + 1), i32(n)
    vals = torch.full((n,), float("nan"), dtype=B.torch_dtype, device="cuda")
    counts = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    spt.spt_coo3_to_csf(B, pos0, crd0, pos1, crd1, pos2, crd2, vals, counts, B.workspace(spt.SPT_OP_TO_CSF))
    torch.cuda.synchronize()
    n0, n1 = (int(x) for x in counts.cpu().numpy())
    nnz = len(spec.vals)
    g = lambda t, m: t.cpu().numpy()[:m]
    return g(pos0, 2), g(crd0, n0), g(pos1, n0 + 1), g(crd1, n1), g(pos2, n1 + 1), g(crd2, nnz), g(vals, nnz)


def gpu_to_ell(spec, W, misalign=False):
    import torch
    import paper_1804_10112_amd as spt
    A = spt.DeviceTensor(spec, misalign=misalign)
    N = spec.dims[0]
    crd = torch.full((max(W * N, 1),), -7, dtype=torch.int32, device="cuda")
    vals = torch.full((max(W * N, 1),), float("nan"), dtype=A.torch_dtype, device="cuda")
    longest = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    spt.spt_to_ell(A, W, crd, vals, longest, A.workspace(spt.SPT_OP_TO_ELL))
    torch.cuda.synchronize()
    return (crd.cpu().numpy()[:W * N].reshape(W, N), vals.cpu().numpy()[:W * N].reshape(W, N),
            int(longest.item()))


def gpu_to_dia(spec, cap=None):
    import torch
    import paper_1804_10112_amd as spt
    A = spt.DeviceTensor(spec)
    N, M = spec.dims
    cap = N + M if cap is None else cap
    offs = torch.full((max(cap, 1),), 12345, dtype=torch.int32, device="cuda")
    K = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    spt.spt_coo_dia_offsets(A, offs, cap, K, A.workspace(spt.SPT_OP_DIA_OFFSETS))
    torch.cuda.synchronize()
    k = int(K.item())
    kk = min(k, cap)
    vals = torch.full((max(kk * N, 1),), float("nan"), dtype=A.torch_dtype, device="cuda")
    spt.spt_coo_to_dia(A, kk, offs, vals)
    torch.cuda.synchronize()
    return k, offs.cpu().numpy()[:kk], vals.cpu().numpy()[:kk * N].reshape(kk, N)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("nnz", [1, 2047, 2048, 2049, 6000, 150_000])
def test_coo3_to_csf(dtype, nnz):
    dims = (50, 40, 300) if nnz < 100_000 else (12, 9, 30_000)      # the latter: fibres span many chunks
    ci, cj, ck, v = wl.random_coo3_entries(dims, nnz, 1200 + nnz, dtype=dtype, dist="u11", skew=1.4)
    coo = wl.coo3_spec(dims, ci, cj, ck, v)
    ref = oracle.pack_csf(coo)
    got = gpu_to_csf(coo)
    for name, g, r in zip(("pos0", "crd0", "pos1", "crd1", "pos2", "crd2"), got, ref):
        assert np.array_equal(g, r), f"{name} differs"
    assert np.array_equal(got[6].astype(np.float64), ref[6])
    mis = gpu_to_csf(coo, misalign=True)
    assert all(np.array_equal(a, b) for a, b in zip(mis, got))
    if nnz >= 6000:                                                 # and the result feeds MTTKRP on CSF
        packed = wl.csf3_spec(dims, *got[:6], got[6])
        rng = np.random.default_rng(1)
        Cm = rng.uniform(-1, 1, (dims[1], 16)).astype(dtype)
        Dm = rng.uniform(-1, 1, (dims[2], 16)).astype(dtype)
        A, mag = oracle.mttkrp(coo, Cm, Dm)
        assert_close(gpu_mttkrp(packed, Cm, Dm), A, mag, dtype, "mttkrp on the packed CSF")


def test_coo3_to_csf_degenerate():
    e = np.zeros(0, np.int32)
    got = gpu_to_csf(wl.coo3_spec((4, 4, 4), e, e, e, np.zeros(0, np.float32)))
    assert list(got[0]) == [0, 0] and list(got[2]) == [0] and list(got[4]) == [0] and len(got[5]) == 0
    one = gpu_to_csf(wl.coo3_spec((4, 4, 4), [3] * 4, [2] * 4, [0, 1, 2, 3], np.arange(4.0)))   # one fibre
    assert list(one[1]) == [3] and list(one[3]) == [2] and list(one[4]) == [0, 4]
    n = 5000                                                       # every entry its own slice
    i = np.arange(n)
    z = np.zeros(n, int)
    got = gpu_to_csf(wl.coo3_spec((n, 2, 2), i, z, z, np.ones(n)))
    assert np.array_equal(got[1], i) and np.array_equal(got[2], np.arange(n + 1)) and np.array_equal(got[4], np.arange(n + 1))


@pytest.mark.parametrize("source", ["coo", "csr"])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_to_ell(source, dtype):
    N, M = 3000, 2500
    r, c, v = wl.random_coo_entries(N, M, 40_000, seed=1300, dtype=dtype)
    spec = wl.coo_spec(N, M, r, c, v) if source == "coo" else wl.csr_from_sorted_coo(N, M, r, c, v)
    W = int(np.bincount(r, minlength=N).max())
    rc, rv, rl = oracle.pack_ell(spec, W)
    gc, gv, gl = gpu_to_ell(spec, W)
    assert gl == rl == W
    assert np.array_equal(gc, rc) and np.array_equal(gv.astype(np.float64), rv)
    x = wl.dense_vector(M, 3, dtype)
    ref, mag = oracle.spmv(spec, x)
    assert_close(gpu_spmv(wl.ell_spec(N, M, gc, gv), x), ref, mag, dtype, "spmv on the packed ELL")
    # too few slots: tails dropped, the longest row still reported; zero slots: only the report
    gc3, gv3, gl3 = gpu_to_ell(spec, 5)
    rc3, rv3, _ = oracle.pack_ell(spec, 5)
    assert gl3 == W and np.array_equal(gc3, rc3) and np.array_equal(gv3.astype(np.float64), rv3)
    assert gpu_to_ell(spec, 0)[2] == W
    mc, mv, _ = gpu_to_ell(spec, W, misalign=True)
    assert np.array_equal(mc, gc) and np.array_equal(mv, gv)


def test_to_ell_config3_shape_and_empty():
    c3 = wl.config3(N=50_000)
    rc, rv, rl = oracle.pack_ell(c3["csr"], c3["W"])
    gc, gv, gl = gpu_to_ell(c3["csr"], c3["W"])
    assert gl == rl and np.array_equal(gc, rc) and np.array_equal(gv.astype(np.float64), rv)
    e = np.zeros(0, np.int32)
    gc, gv, gl = gpu_to_ell(wl.coo_spec(40, 40, e, e, np.zeros(0, np.float32)), 3)
    assert gl == 0 and np.all(gc == -1) and np.all(gv == 0)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_coo_to_dia(dtype):
    c2 = wl.config2(N=30_000, dtype=dtype)
    coo = wl.coo_spec(*c2["csr"].dims, *c2["entries"]) if "entries" in c2 else None
    if coo is None:
        c, v = oracle.to_coo(c2["csr"])
        coo = wl.coo_spec(*c2["csr"].dims, c[0], c[1], v.astype(dtype))
    ro, rv = oracle.pack_dia(coo)
    k, go, gv = gpu_to_dia(coo)
    assert k == len(ro) == 7 and np.array_equal(go, ro)
    assert np.array_equal(gv.astype(np.float64), rv)
    ref, mag = oracle.spmv(coo, c2["x"])
    N, M = coo.dims
    assert_close(gpu_spmv(wl.dia_spec(N, M, go, gv), c2["x"]), ref, mag, dtype, "spmv on the packed DIA")


def test_coo_to_dia_unordered_rectangular_and_capacity():
    N, M = 300, 450
    r, c, v = wl.random_coo_entries(N, M, 5000, seed=1400, dtype=np.float64, sort=False)
    coo = wl.coo_spec(N, M, r, c, v, ordered=False)
    ro, rv = oracle.pack_dia(coo)
    k, go, gv = gpu_to_dia(coo)
    assert k == len(ro) and np.array_equal(go, ro) and np.array_equal(gv, rv)
    assert go[0] >= -(N - 1) and go[-1] <= M - 1
    k2, go2, gv2 = gpu_to_dia(coo, cap=10)                         # capacity below K: the first 10, K reported
    assert k2 == k and np.array_equal(go2, ro[:10]) and np.array_equal(gv2, rv[:10])
    corners = wl.coo_spec(N, M, [0, N - 1], [M - 1, 0], np.array([1.0, 2.0]))     # extreme offsets
    k3, go3, gv3 = gpu_to_dia(corners)
    assert list(go3) == [-(N - 1), M - 1] and gv3[0, N - 1] == 2.0 and gv3[1, 0] == 1.0
    e = np.zeros(0, np.int32)
    assert gpu_to_dia(wl.coo_spec(N, M, e, e, np.zeros(0)))[0] == 0


def test_pack_errors():
    import torch
    import paper_1804_10112_amd as spt
    r, c, v = wl.random_coo_entries(30, 30, 100, seed=1, dtype=np.float32, sort=False)
    un = spt.DeviceTensor(wl.coo_spec(30, 30, r, c, v, ordered=False))
    i = torch.zeros(3000, dtype=torch.int32, device="cuda")
    f = torch.zeros(3000, device="cuda")
    with pytest.raises(spt.SptError):
        spt.spt_to_ell(un, 3, i, f, i, un.workspace(spt.SPT_OP_TO_ELL))         # unordered COO
    ci, cj, ck, w = wl.random_coo3_entries((5, 5, 5), 50, 2, dtype=np.float32)
    csf = spt.DeviceTensor(wl.csf3_from_sorted_coo((5, 5, 5), ci, cj, ck, w))
    cnt = torch.zeros(2, dtype=torch.int64, device="cuda")
    with pytest.raises(spt.SptError):
        spt.spt_coo3_to_csf(csf, i, i, i, i, i, i, f, cnt, None)
    coo3 = spt.DeviceTensor(wl.coo3_spec((5, 5, 5), ci, cj, ck, w))
    with pytest.raises(spt.SptError) as e:
        spt.spt_coo3_to_csf(coo3, i, i, i, i, i, i, f, cnt, None)
    assert "workspace" in str(e.value)
    with pytest.raises(spt.SptError):
        spt.spt_coo_to_dia(coo3, 1, i, f)


def test_packers_full_size():
    """The benchmark configurations' own layouts as the expected result: config 5's COO packed
    to CSF must equal the generator's CSF arrays (which the CPU tests tie to the oracle's packer),
    config 3's CSR packed to ELL its ELL arrays, config 2's matrix its 7 diagonals."""
    c5 = wl.config5()
    got = gpu_to_csf(c5["coo"])
    for lv, (p_, c_) in zip(c5["csf"].levels, ((got[0], got[1]), (got[2], got[3]), (got[4], got[5]))):
        assert np.array_equal(lv.pos, p_) and np.array_equal(lv.crd, c_)
    assert np.array_equal(got[6], c5["csf"].vals)
    del c5, got
    c3 = wl.config3()
    N = c3["csr"].dims[0]
    gc, gv, gl = gpu_to_ell(c3["csr"], c3["W"])
    ell = c3["ell"]
    assert gl == int(np.diff(c3["csr"].levels[1].pos).max())
    assert np.array_equal(gc.reshape(-1), ell.levels[2].crd) and np.array_equal(gv.reshape(-1), ell.vals)
    del c3
    c2 = wl.config2()
    c, v = oracle.to_coo(c2["csr"])
    N = c2["csr"].dims[0]
    k, go, gv = gpu_to_dia(wl.coo_spec(N, N, c[0], c[1], v))
    dia = c2["dia"]
    assert k == 7 and np.array_equal(go, dia.levels[1].offset)
    want = dia.vals.reshape(7, N).copy()
    for d, o in enumerate(go):                    # cells outside the matrix are zero in a packed DIA
        i = np.arange(N)
        want[d, (i + o < 0) | (i + o >= N)] = 0
    assert np.array_equal(gv, want)


def gpu_to_hashed_rows(spec, W):
    import torch
    import paper_1804_10112_amd as spt
    A = spt.DeviceTensor(spec)
    N = spec.dims[0]
    crd = torch.full((N * W,), 77, dtype=torch.int32, device="cuda")
    vals = torch.full((N * W,), float("nan"), dtype=A.torch_dtype, device="cuda")
    dropped = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    spt.spt_to_hashed_rows(A, W, crd, vals, dropped)
    torch.cuda.synchronize()
    return crd.cpu().numpy().reshape(N, W), vals.cpu().numpy().reshape(N, W), int(dropped.item())


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("ordered", [True, False])
def test_to_hashed_rows_is_a_valid_table(dtype, ordered):
    """Table 3's hashed insert with concurrent lanes: which colliding column takes the earlier
    slot is not fixed, so the table is checked for what is unique (the stored set, the values,
    emptiness elsewhere) and for validity (locate's probe sequence reaches every stored column
    before an empty slot); the packed matrix then multiplies like the original."""
    N, M, W = 3000, 5000, 64
    r, c, v = wl.random_coo_entries(N, M, 60_000, seed=1900, dtype=dtype, sort=ordered)
    coo = wl.coo_spec(N, M, r, c, v, ordered=ordered)
    crd, vals, dropped = gpu_to_hashed_rows(coo, W)
    assert dropped == 0
    rr, qq = np.nonzero(crd >= 0)
    got = np.lexsort((crd[rr, qq], rr))
    want = np.lexsort((c, r))
    assert np.array_equal(rr[got], r[want]) and np.array_equal(crd[rr, qq][got], c[want])
    assert np.array_equal(vals[rr, qq][got], v[want])
    assert np.all(crd[crd < 0] == -1) and np.all(vals[crd < 0] == 0)
    # probe sequence: every slot between col % W and the column's slot (cyclically) is occupied
    start = crd[rr, qq] % W
    dist = (qq - start) % W
    for d in range(1, int(dist.max()) + 1):
        m = dist >= d
        assert np.all(crd[rr[m], (start[m] + d - 1) % W] >= 0)
    ocrd, ovals, odropped = oracle.pack_hashed_rows(coo, W)
    assert odropped == 0 and np.array_equal(np.sort(ocrd, axis=1), np.sort(crd, axis=1))
    packed = wl.TensorSpec((N, M), wl.hashed_rows_from_coo(2, 2, [], [], np.zeros(0, dtype), W).levels, vals.reshape(-1))
    packed.levels[0].N, packed.levels[1].N = N, M
    packed.levels[1].crd = crd.reshape(-1)
    x = wl.dense_vector(M, 3, dtype)
    ref, mag = oracle.spmv(coo, x)
    assert_close(gpu_spmv(packed, x), ref, mag, dtype, "spmv on the packed (dense, hashed) matrix")


def test_to_hashed_rows_collision_free_layout_and_full_rows():
    # distinct residues per row: no collisions, the layout is the oracle's bit for bit
    N, M, W = 50, 64, 64
    r = np.repeat(np.arange(N), 10)
    c = np.tile(np.arange(0, 60, 6), N) + (np.arange(N * 10) // 10) % 4
    v = np.arange(N * 10, dtype=np.float64)
    coo = wl.coo_spec(N, M, r, c, v)
    crd, vals, dropped = gpu_to_hashed_rows(coo, W)
    ocrd, ovals, _ = oracle.pack_hashed_rows(coo, W)
    assert dropped == 0 and np.array_equal(crd, ocrd) and np.array_equal(vals, ovals)
    # six columns for four slots in row 0: two are dropped, the table stays consistent
    rows = np.zeros(6, int)
    cols = np.array([0, 4, 8, 12, 16, 20])
    crd, vals, dropped = gpu_to_hashed_rows(wl.coo_spec(2, 40, rows, cols, np.arange(6.0)), 4)
    assert dropped == 2 and np.count_nonzero(crd[0] >= 0) == 4 and np.all(crd[1] == -1)
    assert set(crd[0]) <= set(cols) and all(vals[0][q] == list(cols).index(crd[0][q]) for q in range(4))


def test_dia_offsets_of_a_matrix_with_ten_million_possible_diagonals():
    """5M x 5M with 3000 entries on 40 diagonals near and far: the flags of all N + M - 1 possible
    offsets are scanned by the device-wide prefix sum in its three-kernel form (more than 2048
    tiles of 4096 values; smaller scans let every workgroup add up the earlier tiles itself)."""
    import torch
    import paper_1804_10112_amd as spt
    N = M = 5_000_000
    rng = np.random.default_rng(31)
    offs = np.unique(np.concatenate([rng.integers(-N + 1, M, 36), [-(N - 1), M - 1, 0, 1]]))
    o = rng.choice(offs, 3000)
    lo, hi = np.maximum(0, -o), np.minimum(N, M - o)
    r = (lo + rng.random(3000) * (hi - lo)).astype(np.int64)
    r = np.minimum(r, hi - 1)
    c = r + o
    order = np.lexsort((c, r))
    r, c, o = r[order], c[order], o[order]
    keep = np.ones(len(r), bool)
    keep[1:] = (r[1:] != r[:-1]) | (c[1:] != c[:-1])
    r, c = r[keep], c[keep]
    A = spt.DeviceTensor(wl.coo_spec(N, M, r, c, np.ones(len(r))))
    cap = 64
    out = torch.full((cap,), 12345, dtype=torch.int32, device="cuda")
    K = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    spt.spt_coo_dia_offsets(A, out, cap, K, A.workspace(spt.SPT_OP_DIA_OFFSETS))
    torch.cuda.synchronize()
    expect = np.unique(c - r)
    assert int(K.item()) == len(expect)
    assert np.array_equal(out.cpu().numpy()[: len(expect)], expect)
