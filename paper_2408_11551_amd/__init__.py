"""MI355X-native blocked SpMM on the matrix units (CSR -> row reordering -> BCSR -> MFMA).

Thin ctypes binding over libsmat.so; the function names are those of include/smat.h.
"""
from .smat import (  # noqa: F401
    SMAT_F16, SMAT_BF16, SmatError, SmatMatrix, lib_path,
    smat_default_options, smat_preprocess, smat_get_dims, smat_get_info, smat_get_layout_info, smat_export_perm, smat_export_col_perm, smat_export_bcsr,
    smat_device_bytes, smat_bind_device, smat_export_device_vals, smat_spmm, smat_spmm_static, smat_destroy,
    smat_last_error, smat_last_kernel, smat_probe_read, smat_probe_read_window, smat_probe_gather, smat_probe_pieces, smat_probe_tile_step, smat_probe_mfma,
    smat_ablation_bytes, smat_ablation_bind, smat_ablation_spmm,
)
