"""ctypes binding of libsmat.so: argument marshalling only, one Python function per C entry point.

Host arrays are numpy arrays, device arrays are torch tensors on a HIP device (torch is used
for device memory and streams, nothing else; it is imported before the library is loaded so
that both share one HIP runtime).  There is no fallback: if the shared library is
missing and cannot be built, importing this module fails.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

SMAT_F16, SMAT_BF16, SMAT_E4M3, SMAT_E5M2, SMAT_I8 = 0, 1, 2, 3, 4
_DTYPES = {"f16": SMAT_F16, "bf16": SMAT_BF16, "e4m3": SMAT_E4M3, "e5m2": SMAT_E5M2, "i8": SMAT_I8}


def _dtype_code(dtype) -> int:
    """Name -> smat_dtype_t; numbers pass through (the library rejects unknown ones)."""
    if isinstance(dtype, str):
        if dtype not in _DTYPES:
            raise ValueError(f"unknown dtype {dtype!r}")
        return _DTYPES[dtype]
    return int(dtype)


def _elem_type(dtype):
    """numpy type carrying one value of A or B."""
    return np.uint8 if _dtype_code(dtype) in (SMAT_E4M3, SMAT_E5M2, SMAT_I8) else np.uint16


_STATUS = {0: "SMAT_OK", 1: "SMAT_ERR_INVALID_ARG", 2: "SMAT_ERR_BAD_CSR", 3: "SMAT_ERR_UNSUPPORTED",
           4: "SMAT_ERR_ALLOC", 5: "SMAT_ERR_NOT_BOUND", 6: "SMAT_ERR_HIP"}


class SmatError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status
        self.status_name = _STATUS.get(status, str(status))


class _Options(ctypes.Structure):
    _fields_ = [("block_h", ctypes.c_int), ("block_w", ctypes.c_int),
                ("reorder", ctypes.c_int), ("tau_permille", ctypes.c_int), ("dense_tiles", ctypes.c_int),
                ("concurrent_streams", ctypes.c_int)]


def lib_path() -> str:
    return _build.OUT


def _load():
    # PyTorch ships its own copy of the HIP runtime.  It has to be in the process before
    # libsmat.so is, so that the library binds to that same copy: device pointers and streams
    # that torch hands over then belong to the runtime the library calls.  (Loaded the other way
    # round, the process holds two runtimes, and the library's may not even find the device.)
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        _build.build()                      # raises if hipcc is missing or the build fails
    lib = ctypes.CDLL(path)
    i64, vp, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    lib.smat_default_options.restype = None
    lib.smat_default_options.argtypes = [ctypes.POINTER(_Options)]
    lib.smat_preprocess.restype = ctypes.c_int
    lib.smat_preprocess.argtypes = [i64, i64, vp, vp, vp, ctypes.c_int, ctypes.POINTER(_Options),
                                    ctypes.POINTER(vp)]
    lib.smat_probe_read.restype = ctypes.c_int
    lib.smat_probe_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.smat_probe_read_window.restype = ctypes.c_int
    lib.smat_probe_read_window.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp, vp]
    lib.smat_probe_gather.restype = ctypes.c_int
    lib.smat_probe_gather.argtypes = [vp, ctypes.c_uint32, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    lib.smat_probe_pieces.restype = ctypes.c_int
    lib.smat_probe_pieces.argtypes = [vp, ctypes.c_uint32, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    lib.smat_probe_tile_step.restype = ctypes.c_int
    lib.smat_probe_tile_step.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp, vp]
    lib.smat_probe_mfma.restype = ctypes.c_int
    lib.smat_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp]
    lib.smat_get_layout_info.restype = ctypes.c_int
    lib.smat_get_layout_info.argtypes = [vp] + [ctypes.POINTER(i64)] * 4
    lib.smat_get_dims.restype = ctypes.c_int
    lib.smat_get_dims.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_int)]
    lib.smat_get_info.restype = ctypes.c_int
    lib.smat_get_info.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64),
                                  ctypes.POINTER(ctypes.c_int)]
    lib.smat_export_perm.restype = ctypes.c_int
    lib.smat_export_perm.argtypes = [vp, vp]
    lib.smat_export_col_perm.restype = ctypes.c_int
    lib.smat_export_col_perm.argtypes = [vp, vp, ctypes.POINTER(i64)]
    lib.smat_export_bcsr.restype = ctypes.c_int
    lib.smat_export_bcsr.argtypes = [vp, vp, vp, vp]
    lib.smat_device_bytes.restype = ctypes.c_int
    lib.smat_device_bytes.argtypes = [vp, ctypes.POINTER(sz)]
    lib.smat_bind_device.restype = ctypes.c_int
    lib.smat_bind_device.argtypes = [vp, vp, sz, vp]
    lib.smat_export_device_vals.restype = ctypes.c_int
    lib.smat_export_device_vals.argtypes = [vp, vp, vp]
    lib.smat_spmm.restype = ctypes.c_int
    lib.smat_spmm.argtypes = [vp, vp, i64, vp, i64, i64, vp]
    lib.smat_spmm_static.restype = ctypes.c_int
    lib.smat_spmm_static.argtypes = [vp, vp, i64, vp, i64, i64, vp]
    lib.smat_ablation_bytes.restype = ctypes.c_int
    lib.smat_ablation_bytes.argtypes = [vp, ctypes.POINTER(sz)]
    lib.smat_ablation_bind.restype = ctypes.c_int
    lib.smat_ablation_bind.argtypes = [vp, vp, sz, vp]
    lib.smat_ablation_spmm.restype = ctypes.c_int
    lib.smat_ablation_spmm.argtypes = [vp, ctypes.c_int, vp, i64, vp, i64, i64, vp]
    lib.smat_destroy.restype = None
    lib.smat_destroy.argtypes = [vp]
    lib.smat_last_error.restype = ctypes.c_char_p
    lib.smat_last_error.argtypes = []
    lib.smat_last_kernel.restype = ctypes.c_char_p
    lib.smat_last_kernel.argtypes = []
    return lib


_lib = _load()


def _check(status: int):
    if status != 0:
        raise SmatError(status, _lib.smat_last_error().decode())


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if hasattr(stream, "cuda_stream"):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def smat_last_error() -> str:
    return _lib.smat_last_error().decode()


def smat_last_kernel() -> str:
    return _lib.smat_last_kernel().decode()


def smat_default_options() -> dict:
    o = _Options()
    _lib.smat_default_options(ctypes.byref(o))
    return {"block_h": o.block_h, "block_w": o.block_w, "reorder": o.reorder, "tau_permille": o.tau_permille,
            "dense_tiles": o.dense_tiles, "concurrent_streams": o.concurrent_streams}


def smat_preprocess(M, K, row_ptr, col_idx, vals_bits, dtype, *, reorder=1, tau_permille=700,
                    block_h=16, block_w=16, dense_tiles=0, concurrent_streams=2) -> int:
    """row_ptr int64[M+1], col_idx int32[nnz], vals_bits uint16[nnz] (uint8 for the 8-bit types)
    (HOST) -> opaque handle."""
    rp, rp_p = _host(row_ptr, np.int64)
    ci, ci_p = _host(col_idx, np.int32)
    vals_bits = np.asarray(vals_bits)
    if vals_bits.dtype.itemsize != np.dtype(_elem_type(dtype)).itemsize:
        raise ValueError(f"vals_bits must hold {np.dtype(_elem_type(dtype)).itemsize}-byte values for dtype {dtype!r}")
    vb, vb_p = _host(vals_bits, _elem_type(dtype))
    if rp.size != M + 1:
        raise ValueError("row_ptr must have M+1 entries")
    nnz = int(rp[-1]) if rp.size else 0
    if ci.size < nnz or vb.size < nnz:
        raise ValueError("col_idx / vals shorter than row_ptr[M]")
    opt = _Options(block_h, block_w, reorder, tau_permille, dense_tiles, concurrent_streams)
    out = ctypes.c_void_p()
    _check(_lib.smat_preprocess(M, K, rp_p, ci_p, vb_p, _dtype_code(dtype), ctypes.byref(opt), ctypes.byref(out)))
    return out.value


def smat_get_dims(h) -> dict:
    """Shape and storage type the handle was made for: {"M", "K", "dtype" (a smat_dtype_t number), "elem_bytes"}."""
    M, K, dt = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int()
    _check(_lib.smat_get_dims(h, ctypes.byref(M), ctypes.byref(K), ctypes.byref(dt)))
    return {"M": M.value, "K": K.value, "dtype": dt.value, "elem_bytes": 1 if dt.value in (SMAT_E4M3, SMAT_E5M2, SMAT_I8) else 2}


def _check_device_operands(h, B, C, N, elem_sizes=(1, 2)):
    """Raises ValueError unless B and C are device tensors on one device that hold what the kernels
    will address for this handle: K rows of N elements of the handle's size in B, M rows of N 4-byte
    elements in C.  The library bounds its loads and stores by M, K, N and the leading dimensions it
    is given, not by the tensors, so this is checked here, before any launch.  Returns (N, ldb, ldc)."""
    dims = smat_get_dims(h)
    if B.dim() != 2 or C.dim() != 2 or B.stride(1) != 1 or C.stride(1) != 1:
        raise ValueError("B and C must be 2-D with unit column stride")
    if dims["elem_bytes"] not in elem_sizes:
        raise ValueError("this call does not take the handle's storage type")
    if B.element_size() != dims["elem_bytes"]:
        raise ValueError(f"B must hold {dims['elem_bytes']}-byte elements for this handle, not {B.element_size()}-byte ones")
    if C.element_size() != 4:
        raise ValueError("C must hold 4-byte elements")
    if N is None:
        N = B.shape[1]
    N = int(N)
    if N > B.shape[1] or N > C.shape[1]:            # a negative N is the library's to refuse
        raise ValueError(f"N = {N} exceeds the columns of B ({B.shape[1]}) or C ({C.shape[1]})")
    if B.shape[0] < dims["K"]:
        raise ValueError(f"B has {B.shape[0]} rows, the matrix has K = {dims['K']} columns")
    if C.shape[0] < dims["M"]:
        raise ValueError(f"C has {C.shape[0]} rows, the matrix has M = {dims['M']} rows")
    ldb = B.stride(0) if B.shape[0] > 1 else max(B.shape[1], N)
    ldc = C.stride(0) if C.shape[0] > 1 else max(C.shape[1], N)
    if (dims["K"] > 1 and ldb < N) or (dims["M"] > 1 and ldc < N):
        raise ValueError("rows of B or C overlap (row stride below N)")
    if not (B.is_cuda and C.is_cuda):
        raise ValueError("B and C must be device tensors")
    if B.device != C.device:
        raise ValueError(f"B is on {B.device} and C on {C.device}")
    return N, ldb, ldc


def smat_get_info(h) -> dict:
    nbr, n_e, n_id = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    used = ctypes.c_int()
    _check(_lib.smat_get_info(h, ctypes.byref(nbr), ctypes.byref(n_e), ctypes.byref(n_id), ctypes.byref(used)))
    return {"n_block_rows": nbr.value, "n_blocks": n_e.value, "n_blocks_identity": n_id.value,
            "used_identity": bool(used.value)}


def smat_get_layout_info(h) -> dict:
    n_packs, vb, tb, nc = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(_lib.smat_get_layout_info(h, ctypes.byref(n_packs), ctypes.byref(vb), ctypes.byref(tb), ctypes.byref(nc)))
    return {"n_packs": n_packs.value, "value_bytes": vb.value, "table_bytes": tb.value, "n_columns": nc.value}


def smat_export_perm(h, M) -> np.ndarray:
    perm = np.empty(M, dtype=np.int32)
    _check(_lib.smat_export_perm(h, perm.ctypes.data_as(ctypes.c_void_p)))
    return perm


def smat_export_col_perm(h, K):
    """(col_perm int32[K] with col_perm[new] = old, number of blocks after the row permutation alone)."""
    q = np.empty(K, dtype=np.int32)
    n_rows = ctypes.c_int64()
    _check(_lib.smat_export_col_perm(h, q.ctypes.data_as(ctypes.c_void_p), ctypes.byref(n_rows)))
    return q, n_rows.value


def smat_export_bcsr(h, with_vals=True, dtype=None):
    """vals come back as uint16 or uint8 bit patterns by the HANDLE's storage type; dtype, if given,
    must name a type of that size (kept for callers that state it)."""
    info = smat_get_info(h)
    elem = np.uint8 if smat_get_dims(h)["elem_bytes"] == 1 else np.uint16
    if dtype is not None and np.dtype(_elem_type(dtype)) != np.dtype(elem):
        raise ValueError(f"dtype {dtype!r} does not have the element size of the handle's storage type")
    row_ptr = np.empty(info["n_block_rows"] + 1, dtype=np.int32)
    col_idx = np.empty(info["n_blocks"], dtype=np.int32)
    vals = np.empty((info["n_blocks"], 16, 16), dtype=elem) if with_vals else None
    _check(_lib.smat_export_bcsr(h, row_ptr.ctypes.data_as(ctypes.c_void_p),
                                 col_idx.ctypes.data_as(ctypes.c_void_p),
                                 vals.ctypes.data_as(ctypes.c_void_p) if with_vals else None))
    return row_ptr, col_idx, vals


def smat_device_bytes(h) -> int:
    n = ctypes.c_size_t()
    _check(_lib.smat_device_bytes(h, ctypes.byref(n)))
    return n.value


def smat_bind_device(h, workspace, stream=None):
    """workspace: torch uint8 tensor on the device, at least smat_device_bytes(h) bytes, 256-byte aligned."""
    _check(_lib.smat_bind_device(h, ctypes.c_void_p(workspace.data_ptr()),
                                 workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def smat_export_device_vals(h, stream=None, dtype=None) -> np.ndarray:
    n_e = smat_get_info(h)["n_blocks"]
    elem = np.uint8 if smat_get_dims(h)["elem_bytes"] == 1 else np.uint16
    if dtype is not None and np.dtype(_elem_type(dtype)) != np.dtype(elem):
        raise ValueError(f"dtype {dtype!r} does not have the element size of the handle's storage type")
    vals = np.empty((n_e, 16, 16), dtype=elem)
    _check(_lib.smat_export_device_vals(h, vals.ctypes.data_as(ctypes.c_void_p), _stream_ptr(stream)))
    return vals


def smat_spmm(h, B, C, N=None, stream=None):
    """B: device tensor [K, >=N] of the handle's element size (2 bytes, or 1 for the 8-bit
    types; the library does not know the tensor's type, the caller must match the handle);
    C: device tensor [M, >=N] of 4-byte elements (float32, int32 for "i8"); rows contiguous.
    Shapes, devices and element sizes are checked against the handle before the call (ValueError)."""
    N, ldb, ldc = _check_device_operands(h, B, C, N)
    _check(_lib.smat_spmm(h, ctypes.c_void_p(B.data_ptr()), ldb, ctypes.c_void_p(C.data_ptr()), ldc, N,
                          _stream_ptr(stream)))


def smat_spmm_static(h, B, C, N=None, stream=None):
    """As smat_spmm, with the partial tiles of split launches in the library's static device array."""
    N, ldb, ldc = _check_device_operands(h, B, C, N)
    _check(_lib.smat_spmm_static(h, ctypes.c_void_p(B.data_ptr()), ldb, ctypes.c_void_p(C.data_ptr()), ldc, N,
                                 _stream_ptr(stream)))


def smat_ablation_bytes(h) -> int:
    n = ctypes.c_size_t()
    _check(_lib.smat_ablation_bytes(h, ctypes.byref(n)))
    return n.value


def smat_ablation_bind(h, area, stream=None):
    """area: torch uint8 tensor on the device, at least smat_ablation_bytes(h) bytes, 256-byte aligned."""
    _check(_lib.smat_ablation_bind(h, ctypes.c_void_p(area.data_ptr()), area.numel() * area.element_size(),
                                   _stream_ptr(stream)))


def smat_ablation_spmm(h, level, B, C, N=None, stream=None):
    """As smat_spmm, through the ablation kernel of the given level (0, 1 or 2)."""
    N, ldb, ldc = _check_device_operands(h, B, C, N, elem_sizes=(2,))
    _check(_lib.smat_ablation_spmm(h, level, ctypes.c_void_p(B.data_ptr()), ldb, ctypes.c_void_p(C.data_ptr()), ldc, N,
                                   _stream_ptr(stream)))


def smat_probe_read(buf, sink, stream=None):
    """buf: device tensor read once end to end; sink: device tensor of >= 4 bytes."""
    _check(_lib.smat_probe_read(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream)))


def smat_probe_read_window(buf, window_bytes, waves, sink, stream=None):
    """buf: device tensor whose first window_bytes every one of `waves` wavefronts reads once."""
    if not buf.is_cuda or not sink.is_cuda or window_bytes > buf.numel() * buf.element_size():
        raise ValueError("smat_probe_read_window: device tensors, and a window inside buf")
    _check(_lib.smat_probe_read_window(ctypes.c_void_p(buf.data_ptr()), window_bytes, waves,
                                       ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream)))


def smat_probe_gather(table, row_bytes, idx, waves, packs, bytes_per_lane, sink, stream=None):
    """table: device bytes of rows; idx: device int32/uint32 tensor [waves * packs * 32] of row numbers."""
    _check(_lib.smat_probe_gather(ctypes.c_void_p(table.data_ptr()), row_bytes, ctypes.c_void_p(idx.data_ptr()),
                                  waves, packs, bytes_per_lane, ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream)))


def smat_probe_pieces(table, row_bytes, idx, waves, per_lane, bytes_per_lane, sink, stream=None, checked=False):
    """table: device bytes of rows; idx: device int32/uint32 tensor [waves * per_lane * 64] of row numbers.
    Unless `checked` (the caller has made this call before with the same table and idx), verifies
    with a device sync that every named row lies inside the table before launching."""
    if idx.numel() < waves * per_lane * 64 or idx.element_size() != 4:
        raise ValueError("smat_probe_pieces: idx holds fewer than waves * per_lane * 64 32-bit row numbers")
    if not checked:
        rows = table.numel() * table.element_size() // row_bytes
        lo, hi = int(idx.min()), int(idx.max())
        if lo < 0 or hi >= rows:
            raise ValueError("smat_probe_pieces: a row number lies outside the table")
    _check(_lib.smat_probe_pieces(ctypes.c_void_p(table.data_ptr()), row_bytes, ctypes.c_void_p(idx.data_ptr()),
                                  waves, per_lane, bytes_per_lane, ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream)))


def smat_probe_tile_step(workgroups, steps, parts, buf, sink, stream=None):
    """buf: device tensor of at least 1 MiB (read only); parts: bit set of the pieces of the tile kernel's step."""
    _check(_lib.smat_probe_tile_step(workgroups, steps, parts, ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                     ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream)))


def smat_probe_mfma(workgroups, iters, sink, stream=None):
    _check(_lib.smat_probe_mfma(workgroups, iters, ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream)))


def smat_destroy(h):
    if h:
        _lib.smat_destroy(h)


class SmatMatrix:
    """Owns a handle and the torch workspace tensor it is bound to (memory plumbing only)."""

    def __init__(self, M, K, row_ptr, col_idx, vals_bits, dtype, *, reorder=1, tau_permille=700,
                 dense_tiles=0, concurrent_streams=2, device="cuda:0", bind=True):
        self.M, self.K, self.dtype = M, K, dtype
        self.handle = smat_preprocess(M, K, row_ptr, col_idx, vals_bits, dtype,
                                      reorder=reorder, tau_permille=tau_permille, dense_tiles=dense_tiles,
                                      concurrent_streams=concurrent_streams)
        self.workspace = None
        self.info = smat_get_info(self.handle)
        if bind:
            self.bind(device)

    def bind(self, device="cuda:0"):
        import torch
        nbytes = smat_device_bytes(self.handle)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        with torch.cuda.device(self.workspace.device):
            smat_bind_device(self.handle, self.workspace)
        return self

    def spmm(self, B, C=None, N=None):
        import torch
        if N is None:
            N = B.shape[1]
        if C is None:
            C = torch.empty((self.M, N), dtype=torch.int32 if _dtype_code(self.dtype) == SMAT_I8 else torch.float32,
                            device=B.device)
        smat_spmm(self.handle, B, C, N)
        return C

    def close(self):
        if self.handle:
            smat_destroy(self.handle)
            self.handle = None
        self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
