"""ctypes front end of the plain-C oracle routines (TEST INFRASTRUCTURE, see smat_ref.c).

The functions mirror smat_ref.py one to one; tests pin each against its Python
twin on small inputs, the full-size configurations then use these.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.OUT
        if not os.path.exists(path):
            path = _build.build()
        lib = ctypes.CDLL(path)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.ref_num_threads.restype = ctypes.c_int
        lib.ref_spmm_f64.restype = None
        lib.ref_spmm_f64.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, vp]
        lib.ref_cluster_from_seed.restype = i64
        lib.ref_cluster_from_seed.argtypes = [i64, vp, vp, i64, i32, vp, vp, i64, vp]
        lib.ref_jaccard_reorder.restype = i64
        lib.ref_jaccard_reorder.argtypes = [i64, vp, vp, i64, i32, vp]
        lib.ref_count_blocks.restype = i64
        lib.ref_count_blocks.argtypes = [i64, vp, vp, i64, vp, i32]
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().ref_num_threads())


def block_pattern_csr(M, K, row_ptr, col_idx, w=16):
    """Row patterns (ascending block columns per row) as a CSR-like pair
    (pat_ptr int64[M+1], pat_idx int32[]); CSR columns ascend inside a row, so the
    block columns do too and duplicates are neighbours."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    bc = np.asarray(col_idx, dtype=np.int64) // w
    rows = np.repeat(np.arange(M, dtype=np.int64), np.diff(row_ptr))
    first = np.ones(bc.size, dtype=bool)
    if bc.size > 1:
        first[1:] = (bc[1:] != bc[:-1]) | (rows[1:] != rows[:-1])
    pat_idx = bc[first].astype(np.int32)
    pat_ptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows[first], minlength=M), out=pat_ptr[1:])
    return pat_ptr, pat_idx


def spmm_ref_c(M, K, N, row_ptr, col_idx, a_val, b, want_abs=True):
    """float64 C = A.B (and S = |A|.|B| when want_abs) via ref_spmm_f64."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    a_val = np.ascontiguousarray(a_val, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64).reshape(K, N)
    c = np.empty((M, N), dtype=np.float64)
    s = np.empty((M, N), dtype=np.float64) if want_abs else None
    _load().ref_spmm_f64(M, K, N, _p(row_ptr), _p(col_idx), _p(a_val), _p(b), _p(c),
                         _p(s) if want_abs else None)
    return c, s


def jaccard_reorder_c(M, pat_ptr, pat_idx, nbc, tau_permille):
    perm = np.empty(M, dtype=np.int32)
    n = _load().ref_jaccard_reorder(M, _p(pat_ptr), _p(pat_idx), nbc, tau_permille, _p(perm))
    if n < 0:
        raise ValueError("ref_jaccard_reorder failed (tau out of range or out of memory)")
    return perm, int(n)


def cluster_from_seed_c(M, pat_ptr, pat_idx, nbc, tau_permille, clustered, v):
    """clustered: uint8[M], updated in place; returns the member rows in merge order."""
    assert clustered.dtype == np.uint8 and clustered.flags.c_contiguous
    in_pc = np.zeros(max(nbc, 1), dtype=np.uint8)
    members = np.empty(M, dtype=np.int32)
    n = _load().ref_cluster_from_seed(M, _p(pat_ptr), _p(pat_idx), nbc, tau_permille,
                                      _p(clustered), _p(in_pc), v, _p(members))
    return members[:n].copy()


def count_blocks_c(M, pat_ptr, pat_idx, nbc, perm, h=16):
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    n = _load().ref_count_blocks(M, _p(pat_ptr), _p(pat_idx), nbc, _p(perm), h)
    if n < 0:
        raise MemoryError
    return int(n)


def choose_perm_c(M, pat_ptr, pat_idx, nbc, tau_permille, reorder=True, h=16):
    """Guarded choice, as smat_ref.choose_perm: (perm, n_e, n_e_identity, used_identity)."""
    ident = np.arange(M, dtype=np.int32)
    n_id = count_blocks_c(M, pat_ptr, pat_idx, nbc, ident, h)
    if not reorder:
        return ident, n_id, n_id, True
    cand, _ = jaccard_reorder_c(M, pat_ptr, pat_idx, nbc, tau_permille)
    n_c = count_blocks_c(M, pat_ptr, pat_idx, nbc, cand, h)
    if n_c < n_id:
        return cand, n_c, n_id, False
    return ident, n_id, n_id, True
