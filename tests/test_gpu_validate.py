"""GPU: spt_validate accepts every well-formed tensor of the test generators and names the
kind of every planted defect (defects are planted in copies of the host arrays; no kernel
other than the checker ever sees them)."""
import copy

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _verdict(spec):
    import torch
    import paper_1804_10112_amd as spt
    T = spt.DeviceTensor(spec)
    err = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    spt.spt_validate(T, err)
    torch.cuda.synchronize()
    n, kinds = err.cpu().tolist()
    return n, kinds


def _specs():
    c1 = wl.config1(N=600, nnz=5000)
    c2 = wl.config2(N=3000)
    c3 = wl.config3(N=3000)
    c4 = wl.config4(N=3000, nnz_target=40_000, max_row=2000)
    c5 = wl.config5(dims=(300, 200, 100), nnz=20_000, rank=4)
    r, c, v = c1["entries"]
    i, j, k, tv = wl.random_coo3_entries((300, 200, 100), 5000, 3, np.float32)
    xc, xv = wl.random_sparse_vector(500, 60, seed=4)
    return {"csr": c1["csr"], "coo": c1["coo"], "dia": c2["dia"], "ell": c3["ell"], "coo_unordered": c4["coo"],
            "coo3": c5["coo"], "csf": c5["csf"],
            "csf_gaps": wl.csf3_with_empty_segments((300, 200, 100), i, j, k, tv, 5, 800, 30),
            "dcsr": wl.dcsr_from_sorted_coo(600, 600, r, c, v), "csc": wl.csc_from_coo(600, 600, r, c, v),
            "hashed_rows": wl.hashed_rows_from_coo(600, 600, r, c, v, 32),
            "bcsr": wl.bcsr_from_coo(600, 600, r, c, v, 4, 2),
            "sparse_vector": wl.sparse_vector_spec(500, xc, xv), "hash_vector": wl.hash_vector_spec(500, xc, xv, 128)}


def test_well_formed_tensors_pass():
    for name, spec in _specs().items():
        assert _verdict(spec) == (0, 0), name


def _broken(spec, level, array, edit):
    bad = copy.deepcopy(spec)
    a = np.array(getattr(bad.levels[level], array), copy=True)
    edit(a)
    setattr(bad.levels[level], array, a)
    return bad


def test_planted_defects_are_named():
    import paper_1804_10112_amd as spt
    S = _specs()

    def swap(a, p):
        a[p], a[p + 1] = a[p + 1], a[p]

    cases = [
        ("csr pos decreases", _broken(S["csr"], 1, "pos", lambda a: a.__setitem__(7, a[9] + 1)), spt.SPT_BAD_POS),
        ("csr pos[0] != 0", _broken(S["csr"], 1, "pos", lambda a: a.__setitem__(0, 1)), spt.SPT_BAD_POS),
        ("csr pos ends early", _broken(S["csr"], 1, "pos", lambda a: a.__setitem__(len(a) - 1, a[-1] - 1)), spt.SPT_BAD_POS_END),
        ("csr column = M", _broken(S["csr"], 1, "crd", lambda a: a.__setitem__(11, 600)), spt.SPT_BAD_CRD),
        ("csr negative column", _broken(S["csr"], 1, "crd", lambda a: a.__setitem__(11, -1)), spt.SPT_BAD_CRD),
        ("coo row too large", _broken(S["coo"], 0, "crd", lambda a: a.__setitem__(len(a) - 1, 4096)), spt.SPT_BAD_CRD),
        ("ell column -2", _broken(S["ell"], 2, "crd", lambda a: a.__setitem__(5, -2)), spt.SPT_BAD_CRD),
        ("csf fibre count wrong", _broken(S["csf"], 2, "pos", lambda a: a.__setitem__(len(a) - 1, a[-1] + 3)), spt.SPT_BAD_POS_END),
        ("csf slice coordinates repeat", _broken(S["csf"], 0, "crd", lambda a: a.__setitem__(3, a[2])), spt.SPT_BAD_ORDER),
        ("hash vector coordinate", _broken(S["hash_vector"], 0, "crd", lambda a: a.__setitem__(int(np.argmax(a >= 0)), 500)), spt.SPT_BAD_CRD),
        ("dia offset beyond the matrix", _broken(S["dia"], 1, "offset", lambda a: a.__setitem__(0, -3000)), spt.SPT_BAD_OFFSET),
    ]
    # order defects need a place where the swap really breaks the order
    crd = np.asarray(S["csr"].levels[1].crd)
    pos = np.asarray(S["csr"].levels[1].pos)
    row = int(np.argmax(np.diff(pos) >= 2))
    cases.append(("csr columns out of order", _broken(S["csr"], 1, "crd", lambda a: swap(a, pos[row])), spt.SPT_BAD_ORDER))
    rows = np.asarray(S["coo"].levels[0].crd)
    p = int(np.argmax(np.diff(rows) > 0))
    cases.append(("coo rows out of order", _broken(S["coo"], 0, "crd", lambda a: swap(a, p)), spt.SPT_BAD_ORDER))
    for what, spec, kind in cases:
        if "dia offset" in what:      # DIA shares one offset array between two levels
            spec.levels[2].offset = spec.levels[1].offset
        n, kinds = _verdict(spec)
        assert n >= 1 and kinds & kind, f"{what}: {n} violations, kinds {kinds}"


def test_host_checkable_inconsistencies_come_back_as_status():
    import torch
    import paper_1804_10112_amd as spt
    S = _specs()
    bad = copy.deepcopy(S["ell"])
    bad.vals = bad.vals[:-1]                     # W * N no longer divides
    bad.levels[2].crd = np.asarray(bad.levels[2].crd)[:-1]
    err = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(spt.SptError):
        spt.spt_validate(spt.DeviceTensor(bad), err)
    with pytest.raises(spt.SptError):
        spt.spt_validate(spt.DeviceTensor(S["csr"]), None)
