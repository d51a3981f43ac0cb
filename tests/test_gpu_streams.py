"""GPU: the library enqueues on the caller's stream, never synchronises or
allocates, so its calls can be captured in a HIP graph and replayed; kernels
without atomics are bit-reproducible from run to run."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import assert_close

pytestmark = pytest.mark.gpu


def test_calls_on_a_side_stream_and_in_a_captured_graph():
    import torch
    import paper_1804_10112_amd as spt
    c1 = wl.config1()
    c5 = wl.config5(dims=(300, 200, 100), nnz=40_000)
    A = spt.DeviceTensor(c1["csr"])
    B = spt.DeviceTensor(c5["coo"])
    x = torch.from_numpy(c1["x"]).cuda()
    Cm, Dm = torch.from_numpy(c5["C"]).cuda(), torch.from_numpy(c5["D"]).cuda()
    y = torch.zeros(4096, dtype=torch.float64, device="cuda")
    Aout = torch.zeros(300, 32, dtype=torch.float32, device="cuda")
    ws_a, ws_b = A.workspace(spt.SPT_OP_SPMV), B.workspace(spt.SPT_OP_MTTKRP, 32)
    ref_y, mag_y = oracle.spmv(c1["csr"], c1["x"])
    ref_A, mag_A = oracle.mttkrp(c5["coo"], c5["C"], c5["D"])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        spt.spt_spmv(A, x, y, ws_a)              # binding passes torch's current stream
        spt.spt_mttkrp(B, Cm, Dm, 32, Aout, ws_b)
    side.synchronize()
    eager_y, eager_A = y.clone(), Aout.clone()
    assert_close(eager_y.cpu().numpy(), ref_y, mag_y, np.float64, "side stream spmv")
    assert_close(eager_A.cpu().numpy(), ref_A, mag_A, np.float32, "side stream mttkrp")

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        spt.spt_spmv(A, x, y, ws_a)
        spt.spt_mttkrp(B, Cm, Dm, 32, Aout, ws_b)
    for rep in range(4):                         # eager work and syncs between the replays
        y.fill_(float("nan"))
        Aout.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager_y), f"replay {rep}: spmv differs from the eager result"
        assert torch.equal(Aout, eager_A), f"replay {rep}: mttkrp differs from the eager result"


def test_kernels_without_atomics_are_bit_reproducible():
    import torch
    import paper_1804_10112_amd as spt
    from gpu_util import gpu_coo_to_csr, gpu_mttkrp, gpu_spmv, gpu_ttv
    c4 = wl.config4(N=30_000, nnz_target=500_000, max_row=20_000, with_sorted=True)
    rs, cs, vs = c4["sorted"]
    for spec in (wl.coo_spec(30_000, 30_000, rs, cs, vs), wl.csr_from_sorted_coo(30_000, 30_000, rs, cs, vs)):
        a, b = gpu_spmv(spec, c4["x"], repeat=2)
        assert np.array_equal(a, b)
    c5 = wl.config5(dims=(2000, 1500, 1000), nnz=300_000)
    for fmt in ("coo", "csf"):
        assert np.array_equal(gpu_ttv(c5[fmt], c5["c"])[2], gpu_ttv(c5[fmt], c5["c"])[2])
        assert np.array_equal(gpu_mttkrp(c5[fmt], c5["C"], c5["D"]), gpu_mttkrp(c5[fmt], c5["C"], c5["D"]))
    p1 = gpu_coo_to_csr(c4["coo"], 0)
    p2 = gpu_coo_to_csr(c4["coo"], 0)
    assert all(np.array_equal(u, v) for u, v in zip(p1, p2))


def test_widening_entry_points_in_a_captured_graph():
    """Conversion, sparse addition, INNERPROD, TTM and the CSF packer enqueue only kernels (their
    counts stay on the device), so a graph of them replays to the eager results bit for bit."""
    import torch
    import paper_1804_10112_amd as spt
    dims = (60, 50, 70)
    bi, bj, bk, bv = wl.random_coo3_entries(dims, 20_000, 1, dtype=np.float32, dist="u11", skew=1.3)
    ci, cj, ck, cv = wl.random_coo3_entries(dims, 15_000, 2, dtype=np.float32, dist="u11")
    B = spt.DeviceTensor(wl.coo3_spec(dims, bi, bj, bk, bv))
    Ct = spt.DeviceTensor(wl.coo3_spec(dims, ci, cj, ck, cv))
    c4 = wl.config4(N=5000, nnz_target=60_000, max_row=3000)
    M = spt.DeviceTensor(c4["coo"])
    nnz_m = len(c4["coo"].vals)
    i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
    cap = 35_000
    outs = {
        "add": [i32(cap), i32(cap), i32(cap), torch.zeros(cap, device="cuda"), torch.zeros(1, dtype=torch.int64, device="cuda")],
        "ip": [torch.zeros(1, device="cuda")],
        "ttm": [i32(20_000), i32(20_000), torch.zeros(20_000, 8, device="cuda"), torch.zeros(1, dtype=torch.int64, device="cuda")],
        "csf": [i32(2), i32(20_000), i32(20_001), i32(20_000), i32(20_001), i32(20_000),
                torch.zeros(20_000, device="cuda"), torch.zeros(2, dtype=torch.int64, device="cuda")],
        "csr": [i32(5001), i32(nnz_m), torch.zeros(nnz_m, dtype=torch.float64, device="cuda")],
    }
    Ck = torch.from_numpy(np.random.default_rng(3).uniform(-1, 1, (8, 70)).astype(np.float32)).cuda()
    ws = {"add": torch.empty(spt.spt_add_workspace_bytes(B, Ct), dtype=torch.uint8, device="cuda"),
          "ip": B.workspace(spt.SPT_OP_INNERPROD), "ttm": B.workspace(spt.SPT_OP_TTM, 8),
          "csf": B.workspace(spt.SPT_OP_TO_CSF), "csr": M.workspace(spt.SPT_OP_COO_TO_CSR)}

    def run_all():
        a = outs["add"]
        spt.spt_add(B, Ct, None, a[0], a[1], a[2], a[3], a[4], ws["add"])
        spt.spt_innerprod(B, Ct, outs["ip"][0], ws["ip"])
        t = outs["ttm"]
        spt.spt_ttm(B, Ck, 8, t[0], t[1], t[2], t[3], ws["ttm"])
        spt.spt_coo3_to_csf(B, *outs["csf"], ws["csf"])
        r = outs["csr"]
        spt.spt_coo_to_csr(M, spt.SPT_ORDER_ROW_COL, r[0], r[1], r[2], ws["csr"])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_all()
    side.synchronize()
    eager = {k: [t.clone() for t in v] for k, v in outs.items()}
    assert int(eager["add"][4].item()) > 20_000 and int(eager["ttm"][3].item()) > 0

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    for rep in range(3):
        for v in outs.values():
            for t in v:
                t.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        n_add, n_fib = int(outs["add"][4].item()), int(outs["ttm"][3].item())
        for k, v in outs.items():
            for j, (t, e) in enumerate(zip(v, eager[k])):
                n = {"add": n_add, "ttm": n_fib}.get(k)
                if n is not None and t.shape[0] >= n and t.dim() >= 1 and t.shape[0] > 2:
                    t, e = t[:n], e[:n]                     # capacity beyond the count is never written
                if k == "csf" and t.shape[0] > 2:
                    continue                                 # compared through their counts below
                assert torch.equal(t, e), f"replay {rep}: {k}[{j}] differs"
        n0, n1 = (int(z) for z in outs["csf"][7].cpu())
        e = eager["csf"]
        assert torch.equal(outs["csf"][1][:n0], e[1][:n0]) and torch.equal(outs["csf"][2][:n0 + 1], e[2][:n0 + 1])
        assert torch.equal(outs["csf"][3][:n1], e[3][:n1]) and torch.equal(outs["csf"][4][:n1 + 1], e[4][:n1 + 1])
        nb = len(bv)
        assert torch.equal(outs["csf"][5][:nb], e[5][:nb]) and torch.equal(outs["csf"][6][:nb], e[6][:nb])


def test_later_entry_points_in_a_captured_graph():
    """Element-wise product (CSR x COO, CSR result), SpMV on BCSR / DCSR / CSC / array-of-structs
    COO, and the two element-wise operations with a dense operand or result: captured once,
    replayed three times with eager work in between, compared with the eager results (bit for bit
    where the kernels add in a fixed order, within the tolerance where they use atomics)."""
    import torch
    import paper_1804_10112_amd as spt
    from gpu_util import assert_close
    N, M = 600, 500
    r1, c1, v1 = wl.random_coo_entries(N, M, 40_000, seed=11, dtype=np.float64)
    r2, c2, v2 = wl.random_coo_entries(N, M, 50_000, seed=12, dtype=np.float64)
    csr = spt.DeviceTensor(wl.csr_from_sorted_coo(N, M, r1, c1, v1))
    coo = spt.DeviceTensor(wl.coo_spec(N, M, r2, c2, v2))
    dcsr = spt.DeviceTensor(wl.dcsr_from_sorted_coo(N, M, r1, c1, v1))
    csc = spt.DeviceTensor(wl.csc_from_coo(N, M, r1, c1, v1))
    aos = spt.DeviceTensor(wl.coo_aos_spec((N, M), (r1, c1), v1))
    blk = wl.random_bcsr(150, 125, 4, 4, 0, 30, seed=13, dtype=np.float64)
    bcsr = spt.DeviceTensor(blk["bcsr"])
    x = torch.from_numpy(wl.dense_vector(M, 14)).cuda()
    xb = torch.from_numpy(blk["x"]).cuda()
    D = torch.from_numpy(np.random.default_rng(15).uniform(-1, 1, (N, M))).cuda()
    f64 = lambda *shape: torch.zeros(*shape, dtype=torch.float64, device="cuda")
    i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
    cap = 40_000
    outs = {"mul": [i32(N + 1), i32(cap), f64(cap), torch.zeros(1, dtype=torch.int64, device="cuda")],
            "y": [f64(N) for _ in range(3)], "y_csc": [f64(N)], "yb": [f64(600)],
            "muld": [f64(len(v1))], "dense": [f64(N, M)]}
    ws = {"mul": torch.empty(spt.spt_add_workspace_bytes(csr, coo), dtype=torch.uint8, device="cuda"),
          "dcsr": dcsr.workspace(spt.SPT_OP_SPMV), "csc": csc.workspace(spt.SPT_OP_SPMV),
          "aos": aos.workspace(spt.SPT_OP_SPMV), "bcsr": bcsr.workspace(spt.SPT_OP_SPMV)}

    def run_all():
        m = outs["mul"]
        spt.spt_mul(csr, coo, m[0], None, m[1], None, m[2], m[3], ws["mul"])
        spt.spt_spmv(dcsr, x, outs["y"][0], ws["dcsr"])
        spt.spt_spmv(aos, x, outs["y"][1], ws["aos"])
        spt.spt_spmv(csr, x, outs["y"][2], ws["dcsr"])         # any workspace large enough will do
        spt.spt_spmv(csc, x, outs["y_csc"][0], ws["csc"])
        spt.spt_spmv(bcsr, xb, outs["yb"][0], ws["bcsr"])
        spt.spt_mul_dense(csr, D, M, outs["muld"][0])
        spt.spt_add_to_dense(csr, coo, outs["dense"][0], M)

    run_all()
    torch.cuda.synchronize()
    eager = {k: [t.clone() for t in v] for k, v in outs.items()}
    n_mul = int(eager["mul"][3].item())
    assert 0 < n_mul < 40_000
    assert torch.equal(eager["y"][0], eager["y"][2])           # DCSR and CSR run the same kernel
    ref = eager["y"][2].cpu().numpy()                          # sorted COO of this size: its own order of additions
    assert_close(eager["y"][1].cpu().numpy(), ref, np.abs(ref) + 1.0, np.float64, "aos coo vs csr")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    for rep in range(3):
        for v in outs.values():
            for t in v:
                t.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert int(outs["mul"][3].item()) == n_mul
        for k, v in outs.items():
            for j, (t, e) in enumerate(zip(v, eager[k])):
                if k == "mul" and j in (1, 2):
                    t, e = t[:n_mul], e[:n_mul]
                if k == "y_csc":                              # binned rows are summed with LDS atomics
                    ref = e.cpu().numpy()
                    assert_close(t.cpu().numpy(), ref, np.abs(ref) + 1.0, np.float64, f"replay {rep} csc")
                else:
                    assert torch.equal(t, e), f"replay {rep}: {k}[{j}] differs"
