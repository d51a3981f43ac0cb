"""ctypes binding of the CPU oracle (oracle.c). TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package; the GPU library never does. `build()` compiles oracle.c with gcc into
liboracle.so next to this file; `lib()` loads it, building first only if no
built library exists.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_SO):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _SO, os.path.join(_HERE, "oracle.c"), "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


class OrcLevel(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mode", C.c_int32), ("N", C.c_int64),
                ("M", C.c_int64), ("pos", C.c_void_p), ("crd", C.c_void_p),
                ("offset", C.c_void_p), ("crd_stride", C.c_int64)]


class OrcTensor(C.Structure):
    _fields_ = [("order", C.c_int32), ("nlevels", C.c_int32), ("is_f64", C.c_int32),
                ("pad", C.c_int32), ("lvl", OrcLevel * 4), ("vals", C.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = _declare(C.CDLL(_SO))
    return _lib


_native = None


def lib_native():
    """The same source built for the machine it runs on, as the CPU baseline is meant to be
    timed: gcc -O3 -march=native -fopenmp, compiled on first use into a temporary directory
    (a library built for another CPU must not travel). Falls back to the portable build, with
    `lib_native.flags` saying which one it is."""
    global _native
    if _native is None:
        import tempfile
        so = os.path.join(tempfile.mkdtemp(prefix="orc_native_"), "liboracle_native.so")
        flags = ["-O3", "-march=native", "-fopenmp"]
        try:
            subprocess.run(["gcc", *flags, "-std=c11", "-fPIC", "-shared", "-o", so,
                            os.path.join(_HERE, "oracle.c"), "-lm"], check=True, capture_output=True)
            _native = _declare(C.CDLL(so))
            lib_native.flags = " ".join(flags)
        except Exception:
            _native = lib()
            lib_native.flags = "-O2 (portable build; the native build failed)"
    return _native


def set_threads(n: int) -> int:
    """Threads of the parallel plain loops in the native build; returns the number in effect."""
    return int(lib_native().orc_set_threads(int(n)))


def _declare(L):
    if True:
        vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
        L.orc_set_threads.restype = i32
        L.orc_set_threads.argtypes = [i32]
        L.orc_level_children.restype = i64
        L.orc_level_children.argtypes = [vp, i64, i64, i64, vp, vp, i64]
        L.orc_hashed_locate.restype = i64
        L.orc_hashed_locate.argtypes = [vp, i64, i64, vp]
        L.orc_count.restype = i64
        L.orc_count.argtypes = [vp]
        L.orc_to_coo.restype = None
        L.orc_to_coo.argtypes = [vp, vp, vp]
        L.orc_spmv.restype = None
        L.orc_spmv.argtypes = [vp, vp, i64, vp, vp]
        L.orc_spmv_sparse_x.restype = None
        L.orc_spmv_sparse_x.argtypes = [vp, vp, i64, vp, vp]
        L.orc_spdm.restype = None
        L.orc_spdm.argtypes = [vp, vp, i32, i64, vp, vp]
        L.orc_plain_spdm_coo.restype = None
        L.orc_plain_spdm_coo.argtypes = [i64, i64, vp, vp, vp, vp, i32, vp, i32]
        L.orc_ttm.restype = C.c_int64
        L.orc_ttm.argtypes = [vp, vp, C.c_int32, C.c_int64, C.c_int64, vp, vp, vp, vp]
        L.orc_pack_csf.restype = C.c_int64
        L.orc_pack_csf.argtypes = [vp] * 10
        L.orc_pack_hashed_rows.restype = C.c_int64
        L.orc_pack_hashed_rows.argtypes = [vp, vp, C.c_int64, vp, vp]
        L.orc_pack_ell.restype = C.c_int64
        L.orc_pack_ell.argtypes = [vp, vp, C.c_int64, vp, vp]
        L.orc_dia_offsets.restype = C.c_int64
        L.orc_dia_offsets.argtypes = [vp, vp, C.c_int64, vp]
        L.orc_pack_dia.restype = None
        L.orc_pack_dia.argtypes = [vp, vp, C.c_int64, vp, vp]
        L.orc_add.restype = C.c_int64
        L.orc_add.argtypes = [vp, vp, vp, C.c_int64, vp, vp, vp]
        L.orc_spmv_blocked.restype = None
        L.orc_spmv_blocked.argtypes = [vp, vp, C.c_int64, C.c_int64, C.c_int64, vp, vp]
        L.orc_mul_dense.restype = None
        L.orc_mul_dense.argtypes = [vp, vp, C.c_int64, C.c_int64, vp]
        L.orc_add_to_dense.restype = None
        L.orc_add_to_dense.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, vp]
        L.orc_mul.restype = C.c_int64
        L.orc_mul.argtypes = [vp, vp, vp, C.c_int64, vp, vp, vp]
        L.orc_innerprod.restype = C.c_double
        L.orc_innerprod.argtypes = [vp, vp, vp, vp]
        L.orc_coo_to_csr.restype = None
        L.orc_coo_to_csr.argtypes = [i64, i64, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        L.orc_ttv.restype = i64
        L.orc_ttv.argtypes = [vp, vp, i64, vp, vp, vp, vp]
        L.orc_mttkrp.restype = None
        L.orc_mttkrp.argtypes = [vp, vp, vp, i32, i64, vp, vp]
        L.orc_plain_spmv_csr.restype = None
        L.orc_plain_spmv_csr.argtypes = [i64, vp, vp, vp, vp, vp, i32]
        L.orc_plain_spmv_coo.restype = None
        L.orc_plain_spmv_coo.argtypes = [i64, i64, vp, vp, vp, vp, vp, i32]
        L.orc_plain_spmv_dia.restype = None
        L.orc_plain_spmv_dia.argtypes = [i64, i64, i64, vp, vp, vp, vp, i32]
        L.orc_plain_spmv_ell.restype = None
        L.orc_plain_spmv_ell.argtypes = [i64, i64, vp, vp, vp, vp, i32]
        L.orc_plain_ttv_coo.restype = i64
        L.orc_plain_ttv_coo.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp, vp, i32]
        L.orc_plain_ttv_csf.restype = None
        L.orc_plain_ttv_csf.argtypes = [i64, vp, vp, vp, vp, vp, i32]
        L.orc_plain_mttkrp_coo.restype = None
        L.orc_plain_mttkrp_coo.argtypes = [i64, i64, vp, vp, vp, vp, vp, vp, i32, vp, i32]
        L.orc_plain_mttkrp_csf.restype = None
        L.orc_plain_mttkrp_csf.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, i32]
    return L


def _ptr(a):
    return None if a is None else a.ctypes.data


def _is_f64(dtype) -> int:
    if dtype == np.float64:
        return 1
    if dtype == np.float32:
        return 0
    raise TypeError(f"oracle supports float32/float64 values, got {dtype}")


class OTensor:
    """Holds an OrcTensor plus the numpy arrays it points into."""

    def __init__(self, spec):
        self.spec = spec
        self.keep = []
        t = OrcTensor()
        t.order = spec.order
        t.nlevels = len(spec.levels)
        t.is_f64 = _is_f64(spec.vals.dtype)
        for k, lv in enumerate(spec.levels):
            o = t.lvl[k]
            o.kind, o.mode, o.N, o.M = lv.kind, lv.mode, lv.N, lv.M
            o.crd_stride = getattr(lv, "crd_stride", 1)
            for name in ("pos", "crd", "offset"):
                a = getattr(lv, name)
                if a is not None:
                    a = np.ascontiguousarray(a, dtype=np.int32)
                    self.keep.append(a)
                    setattr(o, name, a.ctypes.data)
        v = np.ascontiguousarray(spec.vals)
        self.keep.append(v)
        t.vals = v.ctypes.data
        self.c = t

    @property
    def ref(self):
        return C.addressof(self.c)


def _same_dtype(spec, a):
    a = np.ascontiguousarray(a)
    if a.dtype != spec.vals.dtype:
        raise TypeError("dense operand dtype must match the tensor's values")
    return a


def level_children(level_spec, p_parent, i_parent=0, i_grand=0):
    """(coordinates, positions) of the children of one parent, per Table 2."""
    t = OrcLevel()
    keep = []
    t.kind, t.mode, t.N, t.M = level_spec.kind, level_spec.mode, level_spec.N, level_spec.M
    for name in ("pos", "crd", "offset"):
        a = getattr(level_spec, name)
        if a is not None:
            a = np.ascontiguousarray(a, dtype=np.int32)
            keep.append(a)
            setattr(t, name, a.ctypes.data)
    n = lib().orc_level_children(C.addressof(t), p_parent, i_parent, i_grand, None, None, 0)
    oi = np.zeros(max(n, 1), np.int64)
    op = np.zeros(max(n, 1), np.int64)
    lib().orc_level_children(C.addressof(t), p_parent, i_parent, i_grand, _ptr(oi), _ptr(op), n)
    return oi[:n], op[:n]


def hashed_locate(level_spec, p_parent, i):
    t = OrcLevel()
    t.kind, t.mode, t.N, t.M = level_spec.kind, level_spec.mode, level_spec.N, level_spec.M
    crd = np.ascontiguousarray(level_spec.crd, dtype=np.int32)
    t.crd = crd.ctypes.data
    found = C.c_int32(0)
    p = lib().orc_hashed_locate(C.addressof(t), p_parent, i, C.addressof(found))
    return int(p), bool(found.value)


def to_coo(spec):
    """All stored leaves in storage order: (coords[order, n] int64, vals[n] float64)."""
    T = OTensor(spec)
    n = lib().orc_count(T.ref)
    coords = np.zeros((spec.order, max(n, 1)), np.int64)
    vals = np.zeros(max(n, 1), np.float64)
    if n:
        # the C side indexes coords_out[m*count + n]
        coords = np.zeros((spec.order, n), np.int64)
        vals = np.zeros(n, np.float64)
        lib().orc_to_coo(T.ref, _ptr(coords), _ptr(vals))
    return coords[:, :n], vals[:n]


def spmv(spec, x):
    """Reference y = A x as float64, plus the magnitude sum per row."""
    T = OTensor(spec)
    x = _same_dtype(spec, x)
    rows = spec.dims[0]
    y = np.zeros(rows, np.float64)
    mag = np.zeros(rows, np.float64)
    lib().orc_spmv(T.ref, _ptr(x), rows, _ptr(y), _ptr(mag))
    return y, mag


def spmv_blocked(spec, x):
    """Reference y = A x for a blocked matrix stored as a 4th-order tensor with dims
    (block rows, block cols, b1, b2): float64 y of length block rows * b1, plus magnitudes."""
    if spec.order != 4:
        raise ValueError("a blocked matrix is a 4th-order tensor")
    T = OTensor(spec)
    x = _same_dtype(spec, x)
    b1, b2 = spec.dims[2], spec.dims[3]
    if len(x) != spec.dims[1] * b2:
        raise ValueError("x must have block cols * b2 entries")
    rows = spec.dims[0] * b1
    y = np.zeros(rows, np.float64)
    mag = np.zeros(rows, np.float64)
    lib().orc_spmv_blocked(T.ref, _ptr(x), b1, b2, rows, _ptr(y), _ptr(mag))
    return y, mag


def spmv_sparse_x(spec, xspec):
    """Reference y = A x with x a 1st-order tensor (sparse vector or hash map)."""
    T, X = OTensor(spec), OTensor(xspec)
    if spec.vals.dtype != xspec.vals.dtype:
        raise TypeError("x must have the dtype of A")
    rows = spec.dims[0]
    y = np.zeros(rows, np.float64)
    mag = np.zeros(rows, np.float64)
    lib().orc_spmv_sparse_x(T.ref, X.ref, rows, _ptr(y), _ptr(mag))
    return y, mag


def spdm(spec, Cm):
    """Reference A = B C (float64) and the magnitude sums."""
    T = OTensor(spec)
    Cm = _same_dtype(spec, Cm)
    J = Cm.shape[1]
    rows = spec.dims[0]
    A = np.zeros((rows, J), np.float64)
    mag = np.zeros((rows, J), np.float64)
    lib().orc_spdm(T.ref, _ptr(Cm), J, rows, _ptr(A), _ptr(mag))
    return A, mag


def plain_spdm(spec, Cm):
    Cm = _same_dtype(spec, Cm)
    lv = spec.levels
    A = np.zeros((spec.dims[0], Cm.shape[1]), spec.vals.dtype)
    lib().orc_plain_spdm_coo(len(spec.vals), spec.dims[0], _ptr(lv[0].crd), _ptr(lv[1].crd),
                             _ptr(spec.vals), _ptr(Cm), Cm.shape[1], _ptr(A), _is_f64(spec.vals.dtype))
    return A


def innerprod(bspec, cspec):
    """Reference alpha = sum B_ijk C_ijk and the magnitude sum."""
    if tuple(bspec.dims) != tuple(cspec.dims):
        raise ValueError("operands differ in shape")
    TB, TC = OTensor(bspec), OTensor(cspec)
    dims = np.asarray(bspec.dims, np.int64)
    mag = C.c_double(0.0)
    a = lib().orc_innerprod(TB.ref, TC.ref, _ptr(dims), C.addressof(mag))
    return float(a), float(mag.value)


def add(bspec, cspec):
    """Reference A = B + C: (list of coordinate arrays, values, magnitudes), ordered, union."""
    if tuple(bspec.dims) != tuple(cspec.dims):
        raise ValueError("operands differ in shape")
    TB, TC = OTensor(bspec), OTensor(cspec)
    order = len(bspec.dims)
    dims = np.asarray(bspec.dims, np.int64)
    cap = max(lib().orc_count(TB.ref) + lib().orc_count(TC.ref), 1)
    crd = [np.zeros(cap, np.int32) for _ in range(order)]
    ptrs = (C.c_void_p * order)(*[c.ctypes.data for c in crd])
    v = np.zeros(cap, np.float64)
    mag = np.zeros(cap, np.float64)
    n = lib().orc_add(TB.ref, TC.ref, _ptr(dims), cap, ptrs, _ptr(v), _ptr(mag))
    if n < 0:
        raise ValueError("orc_add: unsupported operands")
    return [c[:n] for c in crd], v[:n], mag[:n]


def mul_dense(bspec, D):
    """Reference values of B .* D on B's structure: float64[nvals] (0 where a leaf position holds
    no component). D: dense (N, M) array of B's dtype."""
    T = OTensor(bspec)
    D = np.ascontiguousarray(D)
    if D.dtype != bspec.vals.dtype or D.shape != tuple(bspec.dims):
        raise TypeError("D must be a dense matrix of B's shape and dtype")
    out = np.zeros(max(len(bspec.vals), 1), np.float64)
    lib().orc_mul_dense(T.ref, _ptr(D), D.shape[1], len(bspec.vals), _ptr(out))
    return out[:len(bspec.vals)]


def add_to_dense(bspec, cspec):
    """Reference dense A = B + C: (A[N, M] float64, magnitudes)."""
    if tuple(bspec.dims) != tuple(cspec.dims):
        raise ValueError("operands differ in shape")
    TB, TC = OTensor(bspec), OTensor(cspec)
    N, M = bspec.dims
    A = np.zeros((N, M), np.float64)
    mag = np.zeros((N, M), np.float64)
    lib().orc_add_to_dense(TB.ref, TC.ref, N, M, _ptr(A), _ptr(mag))
    return A, mag


def mul(bspec, cspec):
    """Reference A = B .* C: (list of coordinate arrays, values, magnitudes), ordered, intersection."""
    if tuple(bspec.dims) != tuple(cspec.dims):
        raise ValueError("operands differ in shape")
    TB, TC = OTensor(bspec), OTensor(cspec)
    order = len(bspec.dims)
    dims = np.asarray(bspec.dims, np.int64)
    cap = max(min(lib().orc_count(TB.ref), lib().orc_count(TC.ref)), 1)
    crd = [np.zeros(cap, np.int32) for _ in range(order)]
    ptrs = (C.c_void_p * order)(*[c.ctypes.data for c in crd])
    v = np.zeros(cap, np.float64)
    mag = np.zeros(cap, np.float64)
    n = lib().orc_mul(TB.ref, TC.ref, _ptr(dims), cap, ptrs, _ptr(v), _ptr(mag))
    if n < 0:
        raise ValueError("orc_mul: unsupported operands")
    return [c[:n] for c in crd], v[:n], mag[:n]


def pack_csf(spec):
    """(pos0, crd0, pos1, crd1, pos2, crd2, vals) of the tensor packed as CSF."""
    T = OTensor(spec)
    n = max(lib().orc_count(T.ref), 1)
    dims = np.asarray(spec.dims, np.int64)
    i32 = lambda m: np.zeros(m, np.int32)
    pos0, crd0, pos1, crd1, pos2, crd2 = i32(2), i32(n), i32(n + 1), i32(n), i32(n + 1), i32(n)
    vals = np.zeros(n, np.float64)
    counts = np.zeros(2, np.int64)
    nnz = lib().orc_pack_csf(T.ref, _ptr(dims), _ptr(pos0), _ptr(crd0), _ptr(pos1), _ptr(crd1),
                             _ptr(pos2), _ptr(crd2), _ptr(vals), _ptr(counts))
    if nnz < 0:
        raise ValueError("orc_pack_csf: unsupported tensor")
    n0, n1 = int(counts[0]), int(counts[1])
    return pos0, crd0[:n0], pos1[:n0 + 1], crd1[:n1], pos2[:n1 + 1], crd2[:nnz], vals[:nnz]


def pack_hashed_rows(spec, W):
    """(crd[N, W], vals[N, W], dropped) of the matrix packed as (dense rows, hashed columns)."""
    T = OTensor(spec)
    N = spec.dims[0]
    dims = np.asarray(spec.dims, np.int64)
    crd = np.zeros((N, W), np.int32)
    vals = np.zeros((N, W), np.float64)
    dropped = lib().orc_pack_hashed_rows(T.ref, _ptr(dims), W, _ptr(crd), _ptr(vals))
    return crd, vals, int(dropped)


def pack_ell(spec, W):
    """(crd[W, N], vals[W, N], longest row) of the matrix packed as ELL with W slots."""
    T = OTensor(spec)
    N = spec.dims[0]
    dims = np.asarray(spec.dims, np.int64)
    crd = np.zeros((W, N), np.int32)
    vals = np.zeros((W, N), np.float64)
    longest = lib().orc_pack_ell(T.ref, _ptr(dims), W, _ptr(crd), _ptr(vals))
    return crd, vals, int(longest)


def pack_dia(spec):
    """(offsets[K], vals[K, N]) of the matrix packed as DIA."""
    T = OTensor(spec)
    N, M = spec.dims
    dims = np.asarray(spec.dims, np.int64)
    offsets = np.zeros(N + M, np.int32)
    K = int(lib().orc_dia_offsets(T.ref, _ptr(dims), len(offsets), _ptr(offsets)))
    offsets = np.ascontiguousarray(offsets[:K])
    vals = np.zeros((K, N), np.float64)
    lib().orc_pack_dia(T.ref, _ptr(dims), K, _ptr(offsets), _ptr(vals))
    return offsets, vals


def coo_to_csr(nrows, row, col, vals, order=0):
    row = np.ascontiguousarray(row, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    vals = np.ascontiguousarray(vals)
    nnz = len(row)
    pos = np.zeros(nrows + 1, np.int32)
    crd = np.zeros(nnz, np.int32)
    vout = np.zeros(nnz, vals.dtype)
    perm = np.zeros(nnz, np.int64)
    lib().orc_coo_to_csr(nnz, nrows, _ptr(row), _ptr(col), _ptr(vals), vals.dtype.itemsize,
                         order, _ptr(pos), _ptr(crd), _ptr(vout), _ptr(perm))
    return pos, crd, vout, perm


def ttv(spec, c):
    T = OTensor(spec)
    c = _same_dtype(spec, c)
    cap = max(lib().orc_count(T.ref), 1)
    oi = np.zeros(cap, np.int32)
    oj = np.zeros(cap, np.int32)
    ov = np.zeros(cap, np.float64)
    om = np.zeros(cap, np.float64)
    n = lib().orc_ttv(T.ref, _ptr(c), cap, _ptr(oi), _ptr(oj), _ptr(ov), _ptr(om))
    return oi[:n], oj[:n], ov[:n], om[:n]


def ttm(spec, Cm):
    """Reference TTM: (fibre i, fibre j, values[nfib, K], magnitudes[nfib, K]); Cm is K x L."""
    T = OTensor(spec)
    Cm = _same_dtype(spec, Cm)
    K, L = Cm.shape
    if L != spec.dims[2]:
        raise ValueError("C must be K x dims[2]")
    cap = max(lib().orc_count(T.ref), 1)
    oi = np.zeros(cap, np.int32)
    oj = np.zeros(cap, np.int32)
    ov = np.zeros((cap, K), np.float64)
    om = np.zeros((cap, K), np.float64)
    n = lib().orc_ttm(T.ref, _ptr(Cm), K, L, cap, _ptr(oi), _ptr(oj), _ptr(ov), _ptr(om))
    return oi[:n], oj[:n], ov[:n], om[:n]


def mttkrp(spec, Cm, Dm):
    T = OTensor(spec)
    Cm = _same_dtype(spec, Cm)
    Dm = _same_dtype(spec, Dm)
    J = Cm.shape[1]
    I = spec.dims[0]
    A = np.zeros((I, J), np.float64)
    mag = np.zeros((I, J), np.float64)
    lib().orc_mttkrp(T.ref, _ptr(Cm), _ptr(Dm), J, I, _ptr(A), _ptr(mag))
    return A, mag


# ---- plain per-format loops (native dtype); spec must be the named format ----

def plain_spmv(spec, x, fmt, native=False):
    x = _same_dtype(spec, x)
    f = _is_f64(spec.vals.dtype)
    N, M = spec.dims
    y = np.zeros(N, spec.vals.dtype)
    lv = spec.levels
    L = lib_native() if native else lib()
    if fmt == "csr":
        L.orc_plain_spmv_csr(N, _ptr(lv[1].pos), _ptr(lv[1].crd), _ptr(spec.vals), _ptr(x), _ptr(y), f)
    elif fmt == "coo":
        L.orc_plain_spmv_coo(N, len(spec.vals), _ptr(lv[0].crd), _ptr(lv[1].crd), _ptr(spec.vals),
                             _ptr(x), _ptr(y), f)
    elif fmt == "dia":
        L.orc_plain_spmv_dia(N, M, lv[0].N, _ptr(lv[1].offset), _ptr(spec.vals), _ptr(x), _ptr(y), f)
    elif fmt == "ell":
        L.orc_plain_spmv_ell(N, lv[0].N, _ptr(lv[2].crd), _ptr(spec.vals), _ptr(x), _ptr(y), f)
    else:
        raise ValueError(fmt)
    return y


def plain_ttv(spec, c, fmt, native=False):
    c = _same_dtype(spec, c)
    f = _is_f64(spec.vals.dtype)
    lv = spec.levels
    L = lib_native() if native else lib()
    if fmt == "coo":
        nnz = len(spec.vals)
        oi = np.zeros(max(nnz, 1), np.int32)
        oj = np.zeros(max(nnz, 1), np.int32)
        ov = np.zeros(max(nnz, 1), spec.vals.dtype)
        n = L.orc_plain_ttv_coo(nnz, _ptr(lv[0].crd), _ptr(lv[1].crd), _ptr(lv[2].crd),
                                _ptr(spec.vals), _ptr(c), _ptr(oi), _ptr(oj), _ptr(ov), f)
        return oi[:n], oj[:n], ov[:n]
    nfib = len(lv[1].crd)
    ov = np.zeros(max(nfib, 1), spec.vals.dtype)
    L.orc_plain_ttv_csf(nfib, _ptr(lv[2].pos), _ptr(lv[2].crd), _ptr(spec.vals), _ptr(c), _ptr(ov), f)
    return ov[:nfib]


def plain_mttkrp(spec, Cm, Dm, fmt, native=False):
    Cm = _same_dtype(spec, Cm)
    Dm = _same_dtype(spec, Dm)
    f = _is_f64(spec.vals.dtype)
    J = Cm.shape[1]
    I = spec.dims[0]
    A = np.zeros((I, J), spec.vals.dtype)
    lv = spec.levels
    L = lib_native() if native else lib()
    if fmt == "coo":
        L.orc_plain_mttkrp_coo(len(spec.vals), I, _ptr(lv[0].crd), _ptr(lv[1].crd), _ptr(lv[2].crd),
                               _ptr(spec.vals), _ptr(Cm), _ptr(Dm), J, _ptr(A), f)
    else:
        L.orc_plain_mttkrp_csf(I, _ptr(lv[0].pos), _ptr(lv[0].crd), _ptr(lv[1].pos), _ptr(lv[1].crd),
                               _ptr(lv[2].pos), _ptr(lv[2].crd), _ptr(spec.vals), _ptr(Cm), _ptr(Dm),
                               J, _ptr(A), f)
    return A
