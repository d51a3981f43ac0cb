"""spt: sparse tensor kernels over coordinate-hierarchy level formats on MI355X.

Thin ctypes binding of libspt.so (built from csrc/ by build.py). Every step of
the path runs in the library's HIP kernels; this package only marshals
arguments. There is no CPU fallback: loading fails loudly without the library.
"""
from .binding import (  # noqa: F401
    DeviceTensor, SptError, lib, library_path, spt_coo_to_csr, spt_last_error, spt_mttkrp,
    spt_innerprod, spt_ttm, spt_add, spt_mul, spt_mul_dense, spt_add_to_dense, spt_add_workspace_bytes, spt_coo3_to_csf, spt_to_ell, spt_coo_dia_offsets, spt_coo_to_dia, spt_to_coo, spt_to_hashed_rows, spt_spdm, spt_spmv, spt_spmv_static, spt_validate, spt_spmv_sparse_x, spt_ttv, spt_version, spt_workspace_bytes, spt_probe_read, spt_probe_gather,
    SPT_F32, SPT_F64, SPT_STATIC_SCRATCH_BYTES,
    SPT_BAD_POS, SPT_BAD_POS_END, SPT_BAD_CRD, SPT_BAD_ORDER, SPT_BAD_OFFSET,
    SPT_OP_SPMV, SPT_OP_COO_TO_CSR, SPT_OP_TTV, SPT_OP_MTTKRP, SPT_OP_INNERPROD, SPT_OP_TTM, SPT_OP_TO_CSF, SPT_OP_TO_ELL, SPT_OP_DIA_OFFSETS, SPT_OP_TO_COO, SPT_OP_SPMV_SPARSE_X, SPT_OP_SPDM,
    SPT_ORDER_ROW_COL, SPT_ORDER_ROW_STABLE, SPT_ORDERED, SPT_UNIQUE,
)
