"""Helpers for the GPU parity tests: run the library through its C ABI binding
and compare with the oracle under the stated tolerance."""
import numpy as np

TOL = {np.dtype(np.float64): 1e-12, np.dtype(np.float32): 1e-5}


def assert_close(got, ref, mag, dtype, what=""):
    """|got - ref| <= tol * sum|terms| elementwise (forward-error scale of a sum)."""
    tol = TOL[np.dtype(dtype)]
    got = np.asarray(got, np.float64)
    tiny = np.finfo(np.dtype(dtype)).tiny
    err = np.abs(got - ref)
    bound = tol * mag + tiny
    bad = np.flatnonzero(~(err <= bound))
    assert bad.size == 0, (f"{what}: {bad.size} of {got.size} outside tolerance; first at {bad[:5]}: "
                           f"got {got.ravel()[bad[:5]]} ref {np.asarray(ref).ravel()[bad[:5]]} "
                           f"mag {np.asarray(mag).ravel()[bad[:5]]}")


def gpu_spmv(spec, x, repeat=1, misalign=False):
    import torch
    import paper_1804_10112_amd as spt
    A = spt.DeviceTensor(spec, misalign=misalign)
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    ws = A.workspace(spt.SPT_OP_SPMV)
    outs = []
    for _ in range(repeat):
        rows = spec.dims[0] * (spec.dims[2] if len(spec.dims) == 4 else 1)   # order 4: a blocked matrix
        y = torch.full((rows,), float("nan"), dtype=A.torch_dtype, device="cuda")
        spt.spt_spmv(A, xd, y, ws)
        torch.cuda.synchronize()
        outs.append(y.cpu().numpy())
    return outs[0] if repeat == 1 else outs


def gpu_coo_to_csr(spec, order, misalign=False):
    import torch
    import paper_1804_10112_amd as spt
    A = spt.DeviceTensor(spec, misalign=misalign)
    N, nnz = spec.dims[0], len(spec.vals)
    pos = torch.full((N + 1,), -7, dtype=torch.int32, device="cuda")
    crd = torch.full((max(nnz, 1),), -7, dtype=torch.int32, device="cuda")
    vals = torch.zeros(max(nnz, 1), dtype=A.torch_dtype, device="cuda")
    ws = A.workspace(spt.SPT_OP_COO_TO_CSR)
    spt.spt_coo_to_csr(A, order, pos, crd, vals, ws)
    torch.cuda.synchronize()
    return pos.cpu().numpy(), crd.cpu().numpy()[:nnz], vals.cpu().numpy()[:nnz]


def gpu_ttv(spec, c, misalign=False):
    """Returns (out_i, out_j, out_vals, count) for COO input, (None, None, out_vals, count) for CSF."""
    import torch
    import paper_1804_10112_amd as spt
    B = spt.DeviceTensor(spec, misalign=misalign)
    cd = torch.from_numpy(np.ascontiguousarray(c)).cuda()
    nnz = len(spec.vals)
    is_csf = spec.levels[1].kind == 1
    cap = max(len(spec.levels[1].crd) if is_csf else nnz, 1)
    oi = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
    oj = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
    ov = torch.full((cap,), float("nan"), dtype=B.torch_dtype, device="cuda")
    cnt = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ws = B.workspace(spt.SPT_OP_TTV)
    spt.spt_ttv(B, cd, None if is_csf else oi, None if is_csf else oj, ov, cnt, ws)
    torch.cuda.synchronize()
    n = int(cnt.item())
    if is_csf:
        return None, None, ov.cpu().numpy()[:n], n
    return oi.cpu().numpy()[:n], oj.cpu().numpy()[:n], ov.cpu().numpy()[:n], n


def gpu_mttkrp(spec, Cm, Dm, misalign=False):
    import torch
    import paper_1804_10112_amd as spt
    B = spt.DeviceTensor(spec, misalign=misalign)
    Cd = torch.from_numpy(np.ascontiguousarray(Cm)).cuda()
    Dd = torch.from_numpy(np.ascontiguousarray(Dm)).cuda()
    J = Cm.shape[1]
    A = torch.full((spec.dims[0], J), float("nan"), dtype=B.torch_dtype, device="cuda")
    ws = B.workspace(spt.SPT_OP_MTTKRP, J)
    spt.spt_mttkrp(B, Cd, Dd, J, A, ws)
    torch.cuda.synchronize()
    return A.cpu().numpy()


def gpu_spmv_sparse_x(spec, xspec):
    import torch
    import paper_1804_10112_amd as spt
    A = spt.DeviceTensor(spec)
    X = spt.DeviceTensor(xspec)
    y = torch.full((spec.dims[0],), float("nan"), dtype=A.torch_dtype, device="cuda")
    spt.spt_spmv_sparse_x(A, X, y, A.workspace(spt.SPT_OP_SPMV_SPARSE_X))
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_spdm(spec, Cm):
    import torch
    import paper_1804_10112_amd as spt
    B = spt.DeviceTensor(spec)
    Cd = torch.from_numpy(np.ascontiguousarray(Cm)).cuda()
    J = Cm.shape[1]
    A = torch.full((spec.dims[0], J), float("nan"), dtype=B.torch_dtype, device="cuda")
    spt.spt_spdm(B, Cd, J, A, B.workspace(spt.SPT_OP_SPDM, J))
    torch.cuda.synchronize()
    return A.cpu().numpy()


def gpu_innerprod(bspec, cspec):
    import torch
    import paper_1804_10112_amd as spt
    B, Ct = spt.DeviceTensor(bspec), spt.DeviceTensor(cspec)
    out = torch.full((1,), float("nan"), dtype=B.torch_dtype, device="cuda")
    spt.spt_innerprod(B, Ct, out, B.workspace(spt.SPT_OP_INNERPROD))
    torch.cuda.synchronize()
    return float(out.cpu().numpy()[0])


def gpu_ttm(spec, Cm, is_csf=False, fiber_capacity=None, misalign=False):
    """Returns (fibre i, fibre j, values[nfib, K]); i and j are None for CSF input."""
    import torch
    import paper_1804_10112_amd as spt
    B = spt.DeviceTensor(spec, misalign=misalign)
    Cd = torch.from_numpy(np.ascontiguousarray(Cm)).cuda()
    K = Cm.shape[0]
    cap = len(spec.vals) if fiber_capacity is None else fiber_capacity
    oi = torch.full((max(cap, 1),), -7, dtype=torch.int32, device="cuda")
    oj = torch.full((max(cap, 1),), -7, dtype=torch.int32, device="cuda")
    ov = torch.full((max(cap, 1), K), float("nan"), dtype=B.torch_dtype, device="cuda")
    cnt = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ws = B.workspace(spt.SPT_OP_TTM, K)
    if is_csf:
        spt.spt_ttm(B, Cd, K, None, None, ov, cnt, ws)
    else:
        spt.spt_ttm(B, Cd, K, oi, oj, ov, cnt, ws)
    torch.cuda.synchronize()
    n = int(cnt.item())
    if is_csf:
        return None, None, ov.cpu().numpy()[:n]
    return oi.cpu().numpy()[:n], oj.cpu().numpy()[:n], ov.cpu().numpy()[:n]


def gpu_add(bspec, cspec, fmt, misalign=False, op="add"):
    """fmt (B's, hence the result's) 'coo', 'coo3' or 'csr'; op 'add' or 'mul'. Returns (list of
    index arrays, values): for 'csr' the index arrays are [pos, cols], else the coordinate arrays."""
    import torch
    import paper_1804_10112_amd as spt
    B, Ct = spt.DeviceTensor(bspec, misalign=misalign), spt.DeviceTensor(cspec, misalign=misalign)
    cap = max(len(bspec.vals) + len(cspec.vals), 1)
    i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
    c0, c1, c2 = i32(cap), i32(cap), i32(cap)
    pos = i32(bspec.dims[0] + 1)
    ov = torch.full((cap,), float("nan"), dtype=B.torch_dtype, device="cuda")
    cnt = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ws = torch.empty(spt.spt_add_workspace_bytes(B, Ct), dtype=torch.uint8, device="cuda")
    fn = spt.spt_add if op == "add" else spt.spt_mul
    fn(B, Ct, pos if fmt == "csr" else None, None if fmt == "csr" else c0, c1,
       c2 if fmt == "coo3" else None, ov, cnt, ws)
    torch.cuda.synchronize()
    n = int(cnt.item())
    v = ov.cpu().numpy()[:n]
    if fmt == "csr":
        return [pos.cpu().numpy(), c1.cpu().numpy()[:n]], v
    idx = [c0.cpu().numpy()[:n], c1.cpu().numpy()[:n]]
    if fmt == "coo3":
        idx.append(c2.cpu().numpy()[:n])
    return idx, v
