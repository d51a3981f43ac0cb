"""CPU-only checks of the C ABI: the library loads, exports every symbol that
include/spt.h declares, and the host-side validation / recognition logic
returns the documented statuses without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_1804_10112_amd as spt
from paper_1804_10112_amd import binding as B
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _host_desc(spec):
    """An spt_tensor whose pointers are fake but non-null: host validation only."""
    t = B.SptTensor()
    t.order, t.nlevels = len(spec.dims), len(spec.levels)
    t.dtype = B.SPT_F64 if spec.vals.dtype == np.float64 else B.SPT_F32
    for k, lv in enumerate(spec.levels):
        o = t.level[k]
        o.kind, o.mode, o.N, o.M = lv.kind, lv.mode, lv.N, lv.M
        o.flags = (B.SPT_ORDERED if lv.ordered else 0) | (B.SPT_UNIQUE if lv.unique else 0)
        for name in ("pos", "crd", "offset"):
            if getattr(lv, name) is not None:
                setattr(o, name, 0x1000)
    t.vals = 0x1000
    t.nvals = spec.vals.size
    return t


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "spt.h")).read()
    declared = set(re.findall(r"\b(spt_[a-z_0-9]+)\s*\(", header))
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    lib = spt.lib()
    for name in declared:
        assert getattr(lib, name) is not None
    assert "gfx950" in spt.spt_version()


def test_struct_layout_matches_header(tmp_path):
    assert C.sizeof(B.SptLevel) == 4 * 4 + 2 * 8 + 3 * 8 + 8
    assert C.sizeof(B.SptTensor) == 16 + 4 * C.sizeof(B.SptLevel) + 16
    # the same numbers from the header itself, through the C compiler
    import os
    import subprocess
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "spt.h"\n'
                   'int main(void) { printf("%zu %zu %zu %zu %zu %zu\\n", sizeof(spt_level), sizeof(spt_tensor), '
                   'offsetof(spt_level, crd), offsetof(spt_level, crd_stride), offsetof(spt_tensor, level), '
                   'offsetof(spt_tensor, nvals)); return 0; }\n')
    exe = tmp_path / "layout"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe)], check=True)
    got = [int(t) for t in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [C.sizeof(B.SptLevel), C.sizeof(B.SptTensor), B.SptLevel.crd.offset,
                   B.SptLevel.crd_stride.offset, B.SptTensor.level.offset, B.SptTensor.nvals.offset]


def test_recognised_compositions_have_workspace_sizes():
    c1 = wl.config1(N=64, nnz=200)
    c2 = wl.config2(N=64)
    c3 = wl.config3(N=64)
    c5 = wl.config5(dims=(20, 16, 12), nnz=300, rank=4)
    for spec, op in ((c1["csr"], B.SPT_OP_SPMV), (c1["coo"], B.SPT_OP_SPMV), (c2["dia"], B.SPT_OP_SPMV),
                     (c3["ell"], B.SPT_OP_SPMV), (c1["coo"], B.SPT_OP_COO_TO_CSR),
                     (c5["coo"], B.SPT_OP_TTV), (c5["csf"], B.SPT_OP_TTV),
                     (c5["coo"], B.SPT_OP_MTTKRP), (c5["csf"], B.SPT_OP_MTTKRP)):
        assert spt.spt_workspace_bytes(op, _host_desc(spec), 4) >= 256, spec.name


def test_ttv_workspace_follows_the_kernel_choice():
    """The query depends on the descriptor's sizes alone: below 2^18 stored entries (and for a
    last dimension of which less than a quarter would fit LDS) the chunked kernels' carries per
    2048 entries, from 2^18 on the carries and offsets per 256-entry piece."""
    c5 = wl.config5(dims=(20, 16, 12), nnz=300, rank=4)
    sizes = {}
    for fmt in ("coo", "csf"):
        t = _host_desc(c5[fmt])
        for nvals in ((1 << 18) - 1, 1 << 18, 1 << 24):
            t.nvals = nvals
            if fmt == "csf":
                t.level[2].M = 1000          # fibres
            sizes[fmt, nvals] = spt.spt_workspace_bytes(B.SPT_OP_TTV, t)
        assert sizes[fmt, 1 << 18] > 4 * sizes[fmt, (1 << 18) - 1]      # 8x the carries per entry
        assert sizes[fmt, 1 << 24] > 32 * sizes[fmt, 1 << 18]
        t.level[2].N = 10_000_000                                       # c far beyond LDS: chunked again
        t.nvals = 1 << 18
        assert spt.spt_workspace_bytes(B.SPT_OP_TTV, t) < sizes[fmt, 1 << 18]


def _status(fn, *args):
    try:
        fn(*args)
    except spt.SptError as e:
        return e.status, str(e)
    return 0, ""


def test_invalid_and_unsupported_descriptors():
    c1 = wl.config1(N=64, nnz=200)
    # unknown level kind
    t = _host_desc(c1["csr"])
    t.level[1].kind = 9
    assert _status(spt.spt_workspace_bytes, B.SPT_OP_SPMV, t)[0] == B.SPT_ERR_INVALID_ARG
    # Table 1: a hashed level cannot be ordered
    t = _host_desc(c1["csr"])
    t.level[1].kind = wl.HASHED
    st, msg = _status(spt.spt_workspace_bytes, B.SPT_OP_SPMV, t)
    assert st == B.SPT_ERR_INVALID_ARG and "hashed" in msg
    # hashed, legally flagged: (dense, hashed) has no kernel of its own but SpMV reads any
    # composition's level functions per value: the workspace query succeeds (nothing is launched)
    t.level[1].flags = B.SPT_UNIQUE
    t.level[1].M = 8
    assert spt.spt_workspace_bytes(B.SPT_OP_SPMV, t) >= 256
    assert _status(spt.spt_workspace_bytes, B.SPT_OP_MTTKRP, t)[0] == B.SPT_ERR_INVALID_ARG   # reported through the query
    # compressed level without pos; CSR whose column level has the wrong parent count
    t = _host_desc(c1["csr"])
    t.level[1].pos = None
    assert _status(spt.spt_spmv, t, 0x1000, 0x1000, None, 0)[0] == B.SPT_ERR_INVALID_ARG
    t = _host_desc(c1["csr"])
    t.level[1].M = 7
    assert _status(spt.spt_spmv, t, 0x1000, 0x1000, None, 0)[0] == B.SPT_ERR_INVALID_ARG
    # (compressed, compressed) = DCSR: valid for SpMV and to_coo (any composition), not for the
    # operations with format-specific kernels only
    t = _host_desc(c1["coo"])
    t.level[1].kind = wl.COMPRESSED
    t.level[1].pos = 0x1000
    assert spt.spt_workspace_bytes(B.SPT_OP_SPMV, t) >= 256
    assert spt.spt_workspace_bytes(B.SPT_OP_TO_COO, t) >= 256
    assert _status(spt.spt_coo_to_csr, t, 0, 0x1000, 0x1000, 0x1000, None, 0)[0] == B.SPT_ERR_UNSUPPORTED
    # structurally impossible compositions stay unsupported: an offset level without two levels above
    t = _host_desc(c1["csr"])
    t.level[1].kind = wl.OFFSET
    t.level[1].offset = 0x1000
    assert _status(spt.spt_spmv, t, 0x1000, 0x1000, None, 0)[0] == B.SPT_ERR_UNSUPPORTED
    # a 3rd-order tensor is no operand of SpMV
    c5s = wl.config5(dims=(20, 16, 12), nnz=300, rank=4)
    assert _status(spt.spt_spmv, _host_desc(c5s["coo"]), 0x1000, 0x1000, None, 0)[0] == B.SPT_ERR_UNSUPPORTED
    # a workspace that is not 256-byte aligned is refused before anything is launched
    import ctypes
    t = _host_desc(c1["csr"])
    st = B.lib().spt_spmv(ctypes.byref(t), 0x1000, 0x1000, 0x10010, 1 << 20, None)
    assert st == B.SPT_ERR_INVALID_ARG and "aligned" in B.spt_last_error()
    # null operands, bad order, bad rank, wrong operation for the format
    t = _host_desc(c1["coo"])
    assert _status(spt.spt_spmv, t, None, 0x1000, None, 0)[0] == B.SPT_ERR_INVALID_ARG
    assert _status(spt.spt_coo_to_csr, t, 5, 0x1000, 0x1000, 0x1000, None, 0)[0] == B.SPT_ERR_INVALID_ARG
    assert _status(spt.spt_coo_to_csr, _host_desc(c1["csr"]), 0, 0x1000, 0x1000, 0x1000, None, 0)[0] == B.SPT_ERR_UNSUPPORTED
    c5 = wl.config5(dims=(20, 16, 12), nnz=300, rank=4)
    t5 = _host_desc(c5["coo"])
    assert _status(spt.spt_mttkrp, t5, 0x1000, 0x1000, 0, 0x1000, None, 0)[0] == B.SPT_ERR_INVALID_ARG
    assert _status(spt.spt_mttkrp, _host_desc(c1["coo"]), 0x1000, 0x1000, 4, 0x1000, None, 0)[0] == B.SPT_ERR_UNSUPPORTED
    assert _status(spt.spt_ttv, t5, 0x1000, None, None, 0x1000, None, None, 0)[0] == B.SPT_ERR_INVALID_ARG
    # workspace too small is diagnosed before anything is launched
    t = _host_desc(c1["csr"])
    t.level[1].max_children = 100_000       # declared long rows: the entry-balanced kernel and its carries
    st, msg = _status(spt.spt_spmv, t, 0x1000, 0x1000, None, 0)
    assert st == B.SPT_ERR_WORKSPACE and "workspace" in msg
