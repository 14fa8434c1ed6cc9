"""ctypes front end of the C oracles (hyb_oracle.c, sddmm_oracle.c, rgms_oracle.c; fp64 arithmetic).

All arithmetic lives in the C file; this module only compiles it with gcc,
marshals numpy arrays in and copies the resulting arrays out.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("hyb_oracle.c", "sddmm_oracle.c", "rgms_oracle.c")]
_LIB = os.path.join(_HERE, "liboracle_hyb.so")
_lib = None

_i32p = ctypes.c_void_p


class _CHyb(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32), ("c", ctypes.c_int32),
                ("k", ctypes.c_int32), ("w", ctypes.c_int32),
                ("n_buckets", ctypes.c_int64), ("n_ell_rows", ctypes.c_int64),
                ("n_slots", ctypes.c_int64), ("n_rem_segs", ctypes.c_int64),
                ("n_rem_nnz", ctypes.c_int64),
                ("bucket_row_ptr", ctypes.c_void_p), ("bucket_slot_ptr", ctypes.c_void_p),
                ("ell_row", ctypes.c_void_p), ("ell_col", ctypes.c_void_p),
                ("ell_val", ctypes.c_void_p), ("rem_part_ptr", ctypes.c_void_p),
                ("rem_row", ctypes.c_void_p), ("rem_ptr", ctypes.c_void_p),
                ("rem_col", ctypes.c_void_p), ("rem_val", ctypes.c_void_p)]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, *_SRCS, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_hyb_build.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


@dataclass
class HybArrays:
    """The flat hyb(c,k) arrays, host side (numpy)."""
    n_rows: int
    n_cols: int
    c: int
    k: int
    w: int
    bucket_row_ptr: np.ndarray   # int64 [c*(k+1)+1]
    bucket_slot_ptr: np.ndarray  # int64 [c*(k+1)+1]
    ell_row: np.ndarray          # int32 [R]
    ell_col: np.ndarray          # int32 [S]
    ell_val: np.ndarray          # float32 [S]
    rem_part_ptr: np.ndarray     # int32 [c+1]
    rem_row: np.ndarray          # int32 [M]
    rem_ptr: np.ndarray          # int64 [M+1]
    rem_col: np.ndarray          # int32 [T]
    rem_val: np.ndarray          # float32 [T]

    ARRAY_NAMES = ("bucket_row_ptr", "bucket_slot_ptr", "ell_row", "ell_col", "ell_val",
                   "rem_part_ptr", "rem_row", "rem_ptr", "rem_col", "rem_val")


def _copy(ptr, n, dtype):
    if n == 0:
        return np.zeros(0, dtype=dtype)
    buf = (ctypes.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype, count=n).copy()


def _csr_args(indptr, indices, values):
    indptr = np.ascontiguousarray(indptr, dtype=np.int32)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    values = np.ascontiguousarray(values, dtype=np.float32)
    return indptr, indices, values


def hyb_build(n_rows, n_cols, indptr, indices, values, c, k) -> HybArrays:
    lib = _load()
    indptr, indices, values = _csr_args(indptr, indices, values)
    assert indptr.shape[0] == n_rows + 1
    h = _CHyb()
    rc = lib.oracle_hyb_build(ctypes.c_int32(n_rows), ctypes.c_int32(n_cols),
                              ctypes.c_void_p(indptr.ctypes.data), ctypes.c_void_p(indices.ctypes.data),
                              ctypes.c_void_p(values.ctypes.data), ctypes.c_int32(c), ctypes.c_int32(k),
                              ctypes.byref(h))
    if rc != 0:
        lib.oracle_hyb_free(ctypes.byref(h))
        raise ValueError({1: "invalid argument", 2: "columns not strictly ascending or out of range",
                          4: "out of memory"}.get(rc, f"error {rc}"))
    B = h.n_buckets
    out = HybArrays(
        h.n_rows, h.n_cols, h.c, h.k, h.w,
        _copy(h.bucket_row_ptr, B + 1, np.int64), _copy(h.bucket_slot_ptr, B + 1, np.int64),
        _copy(h.ell_row, h.n_ell_rows, np.int32), _copy(h.ell_col, h.n_slots, np.int32),
        _copy(h.ell_val, h.n_slots, np.float32), _copy(h.rem_part_ptr, h.c + 1, np.int32),
        _copy(h.rem_row, h.n_rem_segs, np.int32), _copy(h.rem_ptr, h.n_rem_segs + 1, np.int64),
        _copy(h.rem_col, h.n_rem_nnz, np.int32), _copy(h.rem_val, h.n_rem_nnz, np.float32))
    lib.oracle_hyb_free(ctypes.byref(h))
    return out


def spmm_csr(n_rows, indptr, indices, values, X, want_abs=True):
    """Y = A X by definition in fp64; also sum_j |a_ij x_jk| when want_abs."""
    lib = _load()
    indptr, indices, values = _csr_args(indptr, indices, values)
    X = np.ascontiguousarray(X, dtype=np.float32)
    feat = X.shape[1]
    Y = np.empty((n_rows, feat), dtype=np.float64)
    S = np.empty((n_rows, feat), dtype=np.float64) if want_abs else None
    lib.oracle_spmm_csr(ctypes.c_int32(n_rows), ctypes.c_void_p(indptr.ctypes.data),
                        ctypes.c_void_p(indices.ctypes.data), ctypes.c_void_p(values.ctypes.data),
                        ctypes.c_void_p(X.ctypes.data), ctypes.c_int32(feat),
                        ctypes.c_void_p(Y.ctypes.data),
                        ctypes.c_void_p(S.ctypes.data if want_abs else None))
    return (Y, S) if want_abs else Y


def spmm_csr_rows(rows, indptr, indices, values, X):
    """Rows `rows` of Y = A X (and of the magnitude sums), fp64."""
    lib = _load()
    indptr, indices, values = _csr_args(indptr, indices, values)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    X = np.ascontiguousarray(X, dtype=np.float32)
    feat = X.shape[1]
    Y = np.empty((rows.shape[0], feat), dtype=np.float64)
    S = np.empty((rows.shape[0], feat), dtype=np.float64)
    lib.oracle_spmm_csr_rows(ctypes.c_int64(rows.shape[0]), ctypes.c_void_p(rows.ctypes.data),
                             ctypes.c_void_p(indptr.ctypes.data), ctypes.c_void_p(indices.ctypes.data),
                             ctypes.c_void_p(values.ctypes.data), ctypes.c_void_p(X.ctypes.data),
                             ctypes.c_int32(feat), ctypes.c_void_p(Y.ctypes.data),
                             ctypes.c_void_p(S.ctypes.data))
    return Y, S


def spmm_hyb(h: HybArrays, X):
    """Y evaluated from the hyb arrays, pads included, fp64."""
    lib = _load()
    X = np.ascontiguousarray(X, dtype=np.float32)
    feat = X.shape[1]
    keep = [np.ascontiguousarray(getattr(h, n)) for n in HybArrays.ARRAY_NAMES]
    ch = _CHyb(h.n_rows, h.n_cols, h.c, h.k, h.w, h.c * (h.k + 1), h.ell_row.shape[0],
               h.ell_col.shape[0], h.rem_row.shape[0], h.rem_col.shape[0],
               *[a.ctypes.data for a in keep])
    Y = np.empty((h.n_rows, feat), dtype=np.float64)
    lib.oracle_spmm_hyb(ctypes.byref(ch), ctypes.c_void_p(X.ctypes.data), ctypes.c_int32(feat),
                        ctypes.c_void_p(Y.ctypes.data))
    return Y


def sddmm_csr(n_rows, indptr, indices, values, X, Yt, want_abs=True):
    """B_values[q] = A_ij * sum_k X[i,k] * Yt[j,k] for every stored (i,j), fp64; also the magnitude sums."""
    lib = _load()
    indptr, indices, values = _csr_args(indptr, indices, values)
    X = np.ascontiguousarray(X, dtype=np.float32)
    Yt = np.ascontiguousarray(Yt, dtype=np.float32)
    assert X.shape[1] == Yt.shape[1] and X.shape[0] == n_rows
    d = X.shape[1]
    B = np.empty(indices.shape[0], dtype=np.float64)
    M = np.empty(indices.shape[0], dtype=np.float64) if want_abs else None
    lib.oracle_sddmm_csr(ctypes.c_int32(n_rows), ctypes.c_void_p(indptr.ctypes.data),
                         ctypes.c_void_p(indices.ctypes.data), ctypes.c_void_p(values.ctypes.data),
                         ctypes.c_void_p(X.ctypes.data), ctypes.c_void_p(Yt.ctypes.data), ctypes.c_int32(d),
                         ctypes.c_void_p(B.ctypes.data), ctypes.c_void_p(M.ctypes.data if want_abs else None))
    return (B, M) if want_abs else B


def rgms(n_rel, n_rows, indptr, indices, values, X, W, want_abs=True):
    """Y[i,l] = sum_r sum_j sum_k A[r,i,j] X[j,k] W[r,k,l] in fp64; A stacked slice after slice in CSR."""
    lib = _load()
    indptr, indices, values = _csr_args(indptr, indices, values)
    assert indptr.shape[0] == n_rel * n_rows + 1
    X = np.ascontiguousarray(X, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    assert W.ndim == 3 and W.shape[0] == n_rel and W.shape[1] == X.shape[1]
    d_in, d_out = W.shape[1], W.shape[2]
    Y = np.empty((n_rows, d_out), dtype=np.float64)
    S = np.empty((n_rows, d_out), dtype=np.float64) if want_abs else None
    lib.oracle_rgms(ctypes.c_int32(n_rel), ctypes.c_int32(n_rows), ctypes.c_void_p(indptr.ctypes.data),
                    ctypes.c_void_p(indices.ctypes.data), ctypes.c_void_p(values.ctypes.data),
                    ctypes.c_void_p(X.ctypes.data), ctypes.c_void_p(W.ctypes.data), ctypes.c_int32(d_in),
                    ctypes.c_int32(d_out), ctypes.c_void_p(Y.ctypes.data),
                    ctypes.c_void_p(S.ctypes.data if want_abs else None))
    return (Y, S) if want_abs else Y


def num_threads() -> int:
    return int(_load().oracle_num_threads())
