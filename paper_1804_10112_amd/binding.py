"""ctypes binding of the C ABI declared in include/spt.h (same names).

PyTorch is used for device memory and streams only. `DeviceTensor` uploads the
level arrays of a format description (any object with .dims, .levels[] having
kind/mode/N/M/pos/crd/offset/ordered/unique, and .vals) and packs the pointers
into an spt_tensor struct.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libspt.so")
_lib = None

SPT_OK, SPT_ERR_INVALID_ARG, SPT_ERR_UNSUPPORTED, SPT_ERR_WORKSPACE, SPT_ERR_DEVICE = range(5)
SPT_OP_SPMV, SPT_OP_COO_TO_CSR, SPT_OP_TTV, SPT_OP_MTTKRP, SPT_OP_INNERPROD, SPT_OP_TTM = range(6)
SPT_OP_TO_CSF, SPT_OP_TO_ELL, SPT_OP_DIA_OFFSETS, SPT_OP_TO_COO = 6, 7, 8, 9
SPT_OP_SPMV_SPARSE_X, SPT_OP_SPDM = 10, 11
SPT_ORDER_ROW_COL, SPT_ORDER_ROW_STABLE = 0, 1
SPT_ORDERED, SPT_UNIQUE = 1, 2
SPT_F32, SPT_F64 = 0, 1
SPT_STATIC_SCRATCH_BYTES = 4 << 20

SYMBOLS = ["spt_spmv", "spt_coo_to_csr", "spt_ttv", "spt_mttkrp", "spt_workspace_bytes",
           "spt_last_error", "spt_version", "spt_probe_read", "spt_probe_gather",
           "spt_spmv_sparse_x", "spt_spdm", "spt_innerprod", "spt_ttm",
           "spt_add", "spt_mul", "spt_add_workspace_bytes", "spt_mul_dense", "spt_add_to_dense", "spt_coo3_to_csf", "spt_to_ell",
           "spt_coo_dia_offsets", "spt_coo_to_dia", "spt_to_coo", "spt_to_hashed_rows", "spt_spmv_static", "spt_validate"]


class SptLevel(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mode", C.c_int32), ("flags", C.c_int32),
                ("max_children", C.c_int32), ("N", C.c_int64), ("M", C.c_int64),
                ("pos", C.c_void_p), ("crd", C.c_void_p), ("offset", C.c_void_p),
                ("crd_stride", C.c_int64)]


class SptTensor(C.Structure):
    _fields_ = [("order", C.c_int32), ("nlevels", C.c_int32), ("dtype", C.c_int32),
                ("reserved", C.c_int32), ("level", SptLevel * 4), ("vals", C.c_void_p),
                ("nvals", C.c_int64)]


class SptError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"spt status {status}: {message}")
        self.status = status


def library_path() -> str:
    return _SO


def lib():
    """Loads libspt.so; builds it first only if it has never been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            from . import build as _build
            _build.build()
        L = C.CDLL(_SO)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.spt_spmv.restype = i32
        L.spt_spmv.argtypes = [vp, vp, vp, vp, sz, vp]
        L.spt_validate.restype = i32
        L.spt_validate.argtypes = [vp, vp, vp]
        L.spt_spmv_static.restype = i32
        L.spt_spmv_static.argtypes = [vp, vp, vp, vp]
        L.spt_spmv_sparse_x.restype = i32
        L.spt_spmv_sparse_x.argtypes = [vp, vp, vp, vp, sz, vp]
        L.spt_coo_to_csr.restype = i32
        L.spt_coo_to_csr.argtypes = [vp, i32, vp, vp, vp, vp, sz, vp]
        L.spt_ttv.restype = i32
        L.spt_ttv.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.spt_mttkrp.restype = i32
        L.spt_mttkrp.argtypes = [vp, vp, vp, i32, vp, vp, sz, vp]
        L.spt_coo3_to_csf.restype = i32
        L.spt_coo3_to_csf.argtypes = [vp] * 10 + [sz, vp]
        L.spt_to_ell.restype = i32
        L.spt_to_ell.argtypes = [vp, i32, vp, vp, vp, vp, sz, vp]
        L.spt_coo_dia_offsets.restype = i32
        L.spt_coo_dia_offsets.argtypes = [vp, vp, C.c_int64, vp, vp, sz, vp]
        L.spt_coo_to_dia.restype = i32
        L.spt_coo_to_dia.argtypes = [vp, i32, vp, vp, vp]
        L.spt_to_hashed_rows.restype = i32
        L.spt_to_hashed_rows.argtypes = [vp, i32, vp, vp, vp, vp]
        L.spt_to_coo.restype = i32
        L.spt_to_coo.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.spt_add.restype = i32
        L.spt_add.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.spt_mul.restype = i32
        L.spt_mul.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.spt_mul_dense.restype = i32
        L.spt_mul_dense.argtypes = [vp, vp, C.c_int64, vp, vp]
        L.spt_add_to_dense.restype = i32
        L.spt_add_to_dense.argtypes = [vp, vp, vp, C.c_int64, vp]
        L.spt_add_workspace_bytes.restype = sz
        L.spt_add_workspace_bytes.argtypes = [vp, vp]
        L.spt_ttm.restype = i32
        L.spt_ttm.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.spt_innerprod.restype = i32
        L.spt_innerprod.argtypes = [vp, vp, vp, vp, sz, vp]
        L.spt_spdm.restype = i32
        L.spt_spdm.argtypes = [vp, vp, i32, vp, vp, sz, vp]
        L.spt_workspace_bytes.restype = sz
        L.spt_workspace_bytes.argtypes = [i32, vp, i32]
        L.spt_last_error.restype = C.c_char_p
        L.spt_last_error.argtypes = []
        L.spt_version.restype = C.c_char_p
        L.spt_version.argtypes = []
        L.spt_probe_read.restype = i32
        L.spt_probe_read.argtypes = [vp, sz, i32, vp, vp]
        L.spt_probe_gather.restype = i32
        L.spt_probe_gather.argtypes = [vp, C.c_int64, vp, i32, vp, vp]
        _lib = L
    return _lib


def spt_last_error() -> str:
    return lib().spt_last_error().decode()


def spt_version() -> str:
    return lib().spt_version().decode()


def _check(status):
    if status != SPT_OK:
        raise SptError(status, spt_last_error())


def _p(t):
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _desc(T):
    return C.addressof(T.c) if isinstance(T, DeviceTensor) else C.addressof(T)


def _stream(stream):
    """hipStream_t as an integer; None = torch's current stream (null stream without a GPU)."""
    if stream is None:
        import torch
        if not torch.cuda.is_available():
            return None
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _ws(ws):
    if ws is None or isinstance(ws, int):
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def spt_workspace_bytes(op, T, J=0) -> int:
    n = lib().spt_workspace_bytes(op, _desc(T), J)
    if n == 0:
        raise SptError(SPT_ERR_INVALID_ARG, spt_last_error())
    return n


def spt_spmv(A, x, y, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_spmv(_desc(A), _p(x), _p(y), p, n, _stream(stream)))


SPT_BAD_POS, SPT_BAD_POS_END, SPT_BAD_CRD, SPT_BAD_ORDER, SPT_BAD_OFFSET = 1, 2, 4, 8, 16


def spt_validate(T, err_dev, stream=None):
    _check(lib().spt_validate(_desc(T), _p(err_dev), _stream(stream)))


def spt_spmv_static(A, x, y, stream=None):
    _check(lib().spt_spmv_static(_desc(A), _p(x), _p(y), _stream(stream)))


def spt_spmv_sparse_x(A, x, y, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_spmv_sparse_x(_desc(A), _desc(x), _p(y), p, n, _stream(stream)))


def spt_coo_to_csr(A, order, pos_out, crd_out, vals_out, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_coo_to_csr(_desc(A), order, _p(pos_out), _p(crd_out), _p(vals_out), p, n,
                                _stream(stream)))


def spt_ttv(B, c, out_crd0, out_crd1, out_vals, out_nnz_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_ttv(_desc(B), _p(c), _p(out_crd0), _p(out_crd1), _p(out_vals),
                         _p(out_nnz_dev), p, n, _stream(stream)))


def spt_mttkrp(B, Cm, Dm, J, A_out, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_mttkrp(_desc(B), _p(Cm), _p(Dm), J, _p(A_out), p, n, _stream(stream)))


def spt_probe_read(src, nbytes, lane_bytes, sink, stream=None):
    _check(lib().spt_probe_read(_p(src), nbytes, lane_bytes, _p(sink), _stream(stream)))


def spt_probe_gather(idx, n, table, dtype, out, stream=None):
    _check(lib().spt_probe_gather(_p(idx), n, _p(table), dtype, _p(out), _stream(stream)))


def spt_spdm(B, Cm, J, A_out, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_spdm(_desc(B), _p(Cm), J, _p(A_out), p, n, _stream(stream)))


def spt_ttm(B, Cm, K, out_crd0, out_crd1, out_vals, out_nfib_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_ttm(_desc(B), _p(Cm), K, _p(out_crd0), _p(out_crd1), _p(out_vals),
                         _p(out_nfib_dev), p, n, _stream(stream)))


def spt_coo3_to_csf(B, pos0, crd0, pos1, crd1, pos2, crd2, vals_out, counts_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_coo3_to_csf(_desc(B), _p(pos0), _p(crd0), _p(pos1), _p(crd1), _p(pos2), _p(crd2),
                                 _p(vals_out), _p(counts_dev), p, n, _stream(stream)))


def spt_to_ell(A, W, crd_out, vals_out, longest_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_to_ell(_desc(A), W, _p(crd_out), _p(vals_out), _p(longest_dev), p, n,
                            _stream(stream)))


def spt_coo_dia_offsets(A, offsets_out, cap, K_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_coo_dia_offsets(_desc(A), _p(offsets_out), cap, _p(K_dev), p, n, _stream(stream)))


def spt_coo_to_dia(A, K, offsets, vals_out, stream=None):
    _check(lib().spt_coo_to_dia(_desc(A), K, _p(offsets), _p(vals_out), _stream(stream)))


def spt_to_hashed_rows(A, W, crd_out, vals_out, dropped_dev, stream=None):
    _check(lib().spt_to_hashed_rows(_desc(A), W, _p(crd_out), _p(vals_out), _p(dropped_dev),
                                    _stream(stream)))


def spt_to_coo(T, out_crd0, out_crd1, out_crd2, out_vals, out_nnz_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_to_coo(_desc(T), _p(out_crd0), _p(out_crd1), _p(out_crd2), _p(out_vals),
                            _p(out_nnz_dev), p, n, _stream(stream)))


def spt_add(B, Ct, out_pos, out_crd0, out_crd1, out_crd2, out_vals, out_nnz_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_add(_desc(B), _desc(Ct), _p(out_pos), _p(out_crd0), _p(out_crd1), _p(out_crd2),
                         _p(out_vals), _p(out_nnz_dev), p, n, _stream(stream)))


def spt_mul(B, Ct, out_pos, out_crd0, out_crd1, out_crd2, out_vals, out_nnz_dev, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_mul(_desc(B), _desc(Ct), _p(out_pos), _p(out_crd0), _p(out_crd1), _p(out_crd2),
                         _p(out_vals), _p(out_nnz_dev), p, n, _stream(stream)))


def spt_mul_dense(B, D, ld, out_vals, stream=None):
    _check(lib().spt_mul_dense(_desc(B), _p(D), ld, _p(out_vals), _stream(stream)))


def spt_add_to_dense(B, Ct, A, ld, stream=None):
    _check(lib().spt_add_to_dense(_desc(B), _desc(Ct), _p(A), ld, _stream(stream)))


def spt_add_workspace_bytes(B, Ct):
    n = lib().spt_add_workspace_bytes(_desc(B), _desc(Ct))
    if n == 0:
        raise SptError(SPT_ERR_INVALID_ARG, spt_last_error())
    return n


def spt_innerprod(B, Ct, alpha_out, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().spt_innerprod(_desc(B), _desc(Ct), _p(alpha_out), p, n, _stream(stream)))


class DeviceTensor:
    """spt_tensor descriptor whose level arrays live in device memory."""

    def __init__(self, spec, device="cuda:0", misalign=False):
        """misalign=True places every array one element past a 256-byte boundary
        (exercises the kernels' paths for buffers that are not 16-byte aligned)."""
        import torch
        self.spec = spec
        self.device = device
        self.keep = []
        t = SptTensor()
        t.order = len(spec.dims)
        t.nlevels = len(spec.levels)
        vals = np.ascontiguousarray(spec.vals)
        if vals.dtype == np.float64:
            t.dtype = SPT_F64
        elif vals.dtype == np.float32:
            t.dtype = SPT_F32
        else:
            raise TypeError(f"values must be float32 or float64, got {vals.dtype}")
        shared = {}
        for k, lv in enumerate(spec.levels):
            o = t.level[k]
            o.kind, o.mode, o.N, o.M = int(lv.kind), int(lv.mode), int(lv.N), int(lv.M)
            o.flags = (SPT_ORDERED if lv.ordered else 0) | (SPT_UNIQUE if lv.unique else 0)
            o.max_children = int(getattr(lv, "max_children", 0))
            o.crd_stride = int(getattr(lv, "crd_stride", 1))
            for name in ("pos", "crd", "offset"):
                a = getattr(lv, name)
                if a is None:
                    continue
                if name == "crd" and o.crd_stride > 1 and a.base is not None:
                    # interleaved coordinates: the levels are views into one array, which is
                    # uploaded once; each level points at its own first element of it
                    base = a.base
                    if id(base) not in shared:
                        d = self._upload(np.ascontiguousarray(base, dtype=np.int32).reshape(-1), device, misalign)
                        shared[id(base)] = d
                        self.keep.append(d)
                        setattr(self, "crd_interleaved", d)
                    off = a.__array_interface__["data"][0] - base.__array_interface__["data"][0]
                    o.crd = shared[id(base)].data_ptr() + off
                    continue
                if id(a) not in shared:   # DIA shares one offset array between two levels
                    d = self._upload(np.ascontiguousarray(a, dtype=np.int32), device, misalign)
                    shared[id(a)] = d
                    self.keep.append(d)
                    setattr(self, f"{name}{k}", d)
                setattr(o, name, shared[id(a)].data_ptr())
        self.vals = self._upload(vals, device, misalign)
        t.vals = self.vals.data_ptr()
        t.nvals = vals.size
        self.torch_dtype = self.vals.dtype
        self.c = t

    @staticmethod
    def _upload(a, device, misalign):
        import torch
        if not misalign:
            return torch.from_numpy(a).to(device)
        buf = torch.empty(a.size + 1, dtype=torch.from_numpy(a).dtype, device=device)
        buf[1:].copy_(torch.from_numpy(a))
        return buf[1:]

    def workspace(self, op, J=0):
        import torch
        n = spt_workspace_bytes(op, self, J)
        return torch.empty(n, dtype=torch.uint8, device=self.device)
