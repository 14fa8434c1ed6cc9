"""ctypes binding of libsptir.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/sptir.h).
PyTorch supplies device memory (tensors) and streams; all computation happens
inside the HIP library.  There is no CPU fallback: if the library is missing
or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # imported before the library so that both share torch's HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsptir.so")

SPTIR_OK = 0
ARRAY_IDS = {"bucket_row_ptr": 0, "bucket_slot_ptr": 1, "ell_row": 2, "ell_col": 3, "ell_val": 4,
             "rem_part_ptr": 5, "rem_row": 6, "rem_ptr": 7, "rem_col": 8, "rem_val": 9,
             "plan_stream": 100, "plan_rb_chunk_ptr": 101, "plan_rb_order": 102, "plan_hlist_first_slot": 103,
             "plan_row_slot_ptr": 104, "plan_row_slots": 105, "plan_heavy_rows": 106, "plan_row_val": 107}
ARRAY_DTYPES = {"bucket_row_ptr": np.int64, "bucket_slot_ptr": np.int64, "ell_row": np.int32,
                "ell_col": np.int32, "ell_val": np.float32, "rem_part_ptr": np.int32,
                "rem_row": np.int32, "rem_ptr": np.int64, "rem_col": np.int32, "rem_val": np.float32,
                "plan_stream": np.int32, "plan_rb_chunk_ptr": np.int64, "plan_rb_order": np.int32,
                "plan_hlist_first_slot": np.int32, "plan_row_slot_ptr": np.int32, "plan_row_slots": np.int32,
                "plan_heavy_rows": np.int32, "plan_row_val": np.float32}


class SptirError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = sptir_status_string(status)
        if status == 5 or (status == 6 and where == "sptir_spmm_noalloc"):
            detail += ": " + _lib.sptir_last_hip_error().decode()
        super().__init__(f"{where}: {detail} (status {status})")


class _Csr(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32), ("nnz", ctypes.c_int64),
                ("indptr", ctypes.c_void_p), ("indices", ctypes.c_void_p), ("values", ctypes.c_void_p)]


class _Info(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32), ("n_col_parts", ctypes.c_int32),
                ("max_bucket_log2", ctypes.c_int32), ("part_width", ctypes.c_int32),
                ("n_buckets", ctypes.c_int32), ("nnz", ctypes.c_int64), ("n_ell_rows", ctypes.c_int64),
                ("n_ell_slots", ctypes.c_int64), ("n_pad_slots", ctypes.c_int64),
                ("n_rem_pieces", ctypes.c_int64), ("n_rem_nnz", ctypes.c_int64),
                ("n_work_items", ctypes.c_int64), ("item_slots", ctypes.c_int32),
                ("row_block", ctypes.c_int32), ("n_phases", ctypes.c_int32), ("rounds", ctypes.c_int32),
                ("n_heavy_pieces", ctypes.c_int64), ("n_heavy_items", ctypes.c_int64), ("n_heavy_nnz", ctypes.c_int64),
                ("heavy_len", ctypes.c_int32), ("n_heavy_lists", ctypes.c_int32), ("values_per_row", ctypes.c_int32),
                ("compact_stream", ctypes.c_int32), ("n_row_blocks", ctypes.c_int32),
                ("parts_per_launch", ctypes.c_int32), ("device_bytes", ctypes.c_int64),
                ("full_rows", ctypes.c_int32), ("heavy_list_items", ctypes.c_int32)]


class _BuildOptions(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_int32), ("feat_hint", ctypes.c_int32), ("row_block", ctypes.c_int32),
                ("parts_per_launch", ctypes.c_int32), ("rounds", ctypes.c_int32), ("wide_stream", ctypes.c_int32),
                ("heavy_len", ctypes.c_int32), ("sweep_kb", ctypes.c_int32), ("release_canonical", ctypes.c_int32),
                ("no_spmm_plan", ctypes.c_int32), ("keep_values", ctypes.c_int32), ("light_piece_len", ctypes.c_int32),
                ("full_rows", ctypes.c_int32)]


def _options(options):
    """dict of sptir_build_options_t fields -> the struct (None stays None: the library's defaults)."""
    if not options:
        return None
    o = _BuildOptions()
    o.struct_size = ctypes.sizeof(_BuildOptions)
    names = {name for name, _ in _BuildOptions._fields_} - {"struct_size"}
    for key, value in options.items():
        if key not in names:
            raise KeyError(f"unknown build option {key!r}")
        setattr(o, key, int(value))
    return o


class _LaunchPlan(ctypes.Structure):
    _fields_ = [("row_block", ctypes.c_int32), ("parts_per_launch", ctypes.c_int32), ("n_launches", ctypes.c_int32),
                ("compact_stream", ctypes.c_int32), ("n_feature_tiles", ctypes.c_int32),
                ("tiles_per_sweep", ctypes.c_int32), ("n_sweeps", ctypes.c_int32), ("rounds", ctypes.c_int32),
                ("full_rows", ctypes.c_int32)]


class _PlanInfo(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32), ("n_col_parts", ctypes.c_int32),
                ("part_width", ctypes.c_int32), ("nnz", ctypes.c_int64), ("n_runs", ctypes.c_int64),
                ("device_bytes", ctypes.c_int64)]


class _RgmsInfo(ctypes.Structure):
    _fields_ = [("n_relations", ctypes.c_int32), ("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32),
                ("max_bucket_log2", ctypes.c_int32), ("nnz", ctypes.c_int64),
                ("n_stacked_rows_stored", ctypes.c_int64), ("n_pad_slots", ctypes.c_int64),
                ("n_tiles", ctypes.c_int64), ("workspace_d_out", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("device_bytes", ctypes.c_int64)]


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)

_lib = None
_hip = None

class _SpmmTimes(ctypes.Structure):
    _fields_ = [("ms_lists", ctypes.c_float), ("ms_heavy", ctypes.c_float), ("ms_reduce", ctypes.c_float),
                ("n_list_launches", ctypes.c_int32), ("n_heavy_launches", ctypes.c_int32),
                ("n_reduce_launches", ctypes.c_int32)]


EXPORTED_SYMBOLS = ("sptir_spmm_timed", "sptir_roof_gather", "sptir_roof_fma", "sptir_set_allocator", "sptir_release_scratch", "sptir_hyb_build", "sptir_hyb_build_ex", "sptir_hyb_search", "sptir_default_bucket_log2", "sptir_gather_offsets_fit_32", "sptir_spmm",
                    "sptir_spmm_noalloc",
                    "sptir_spmm_csr", "sptir_sddmm_csr", "sptir_sddmm_plan_build", "sptir_sddmm",
                    "sptir_sddmm_plan_info", "sptir_sddmm_plan_destroy", "sptir_rgms_build", "sptir_rgms", "sptir_rgms_info",
                    "sptir_rgms_destroy", "sptir_hyb_destroy", "sptir_hyb_info", "sptir_hyb_array",
                    "sptir_launch_plan", "sptir_sddmm_default_col_parts", "sptir_status_string", "sptir_last_hip_error")


def load_library(path: str | None = None):
    """Loads libsptir.so (built beforehand by paper_2207_04606_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built; run `python -m paper_2207_04606_amd.build` first")
    lib = ctypes.CDLL(path)
    lib.sptir_set_allocator.restype = ctypes.c_int
    lib.sptir_set_allocator.argtypes = [_ALLOC_FN, _FREE_FN, ctypes.c_void_p]
    lib.sptir_hyb_build.restype = ctypes.c_int
    lib.sptir_hyb_build.argtypes = [ctypes.POINTER(_Csr), ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                    ctypes.POINTER(ctypes.c_void_p)]
    lib.sptir_hyb_build_ex.restype = ctypes.c_int
    lib.sptir_hyb_build_ex.argtypes = [ctypes.POINTER(_Csr), ctypes.c_int32, ctypes.c_int32,
                                       ctypes.POINTER(_BuildOptions), ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
    lib.sptir_default_bucket_log2.restype = ctypes.c_int32
    lib.sptir_default_bucket_log2.argtypes = [ctypes.c_int64, ctypes.c_int32]
    lib.sptir_gather_offsets_fit_32.restype = ctypes.c_int32
    lib.sptir_gather_offsets_fit_32.argtypes = [ctypes.c_int64, ctypes.c_int32]
    lib.sptir_spmm.restype = ctypes.c_int
    lib.sptir_spmm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
    lib.sptir_spmm_timed.restype = ctypes.c_int
    lib.sptir_spmm_timed.argtypes = lib.sptir_spmm.argtypes + [ctypes.POINTER(_SpmmTimes)]
    lib.sptir_roof_gather.restype = ctypes.c_int
    lib.sptir_roof_gather.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                      ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
    lib.sptir_roof_fma.restype = ctypes.c_int
    lib.sptir_roof_fma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
    lib.sptir_spmm_noalloc.restype = ctypes.c_int
    lib.sptir_spmm_noalloc.argtypes = lib.sptir_spmm.argtypes
    lib.sptir_sddmm_csr.restype = ctypes.c_int
    lib.sptir_sddmm_csr.argtypes = [ctypes.POINTER(_Csr), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_int32, ctypes.c_void_p]
    lib.sptir_hyb_search.restype = ctypes.c_int
    lib.sptir_hyb_search.argtypes = [ctypes.POINTER(_Csr), ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p),
                                     ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p]
    lib.sptir_sddmm_plan_build.restype = ctypes.c_int
    lib.sptir_sddmm_plan_build.argtypes = [ctypes.POINTER(_Csr), ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                           ctypes.POINTER(ctypes.c_void_p)]
    lib.sptir_sddmm.restype = ctypes.c_int
    lib.sptir_sddmm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                ctypes.c_int32, ctypes.c_void_p]
    lib.sptir_sddmm_plan_info.restype = ctypes.c_int
    lib.sptir_sddmm_plan_info.argtypes = [ctypes.c_void_p, ctypes.POINTER(_PlanInfo)]
    lib.sptir_sddmm_plan_destroy.restype = ctypes.c_int
    lib.sptir_sddmm_plan_destroy.argtypes = [ctypes.c_void_p]
    lib.sptir_rgms_build.restype = ctypes.c_int
    lib.sptir_rgms_build.argtypes = [ctypes.POINTER(_Csr), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
    lib.sptir_rgms.restype = ctypes.c_int
    lib.sptir_rgms.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                               ctypes.c_int32, ctypes.c_void_p]
    lib.sptir_rgms_info.restype = ctypes.c_int
    lib.sptir_rgms_info.argtypes = [ctypes.c_void_p, ctypes.POINTER(_RgmsInfo)]
    lib.sptir_rgms_destroy.restype = ctypes.c_int
    lib.sptir_rgms_destroy.argtypes = [ctypes.c_void_p]
    lib.sptir_spmm_csr.restype = ctypes.c_int
    lib.sptir_spmm_csr.argtypes = [ctypes.POINTER(_Csr), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                   ctypes.c_void_p]
    lib.sptir_hyb_destroy.restype = ctypes.c_int
    lib.sptir_hyb_destroy.argtypes = [ctypes.c_void_p]
    lib.sptir_hyb_info.restype = ctypes.c_int
    lib.sptir_hyb_info.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Info)]
    lib.sptir_hyb_array.restype = ctypes.c_int
    lib.sptir_hyb_array.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p),
                                    ctypes.POINTER(ctypes.c_int64)]
    lib.sptir_sddmm_default_col_parts.restype = ctypes.c_int32
    lib.sptir_sddmm_default_col_parts.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32]
    lib.sptir_launch_plan.restype = ctypes.c_int
    lib.sptir_launch_plan.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                      ctypes.POINTER(_BuildOptions), ctypes.POINTER(_LaunchPlan)]
    lib.sptir_status_string.restype = ctypes.c_char_p
    lib.sptir_status_string.argtypes = [ctypes.c_int]
    lib.sptir_last_hip_error.restype = ctypes.c_char_p
    lib.sptir_last_hip_error.argtypes = []
    _lib = lib
    return lib


def _hip_runtime():
    """The HIP runtime torch already loaded (for device-to-host copies of raw pointers)."""
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL(os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"))
        _hip.hipMemcpy.restype = ctypes.c_int
        _hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    return _hip


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev(t: torch.Tensor, dtype, what: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def _csr_struct(n_rows, n_cols, indptr, indices, values):
    """values may be None where only the structure is read."""
    _dev(indptr, torch.int32, "indptr"); _dev(indices, torch.int32, "indices")
    if values is not None:
        _dev(values, torch.float32, "values")
    if indptr.numel() != n_rows + 1 or (values is not None and indices.numel() != values.numel()):
        raise ValueError("CSR array sizes do not match")
    return _Csr(n_rows, n_cols, indices.numel(), indptr.data_ptr(), indices.data_ptr() or None,
                (values.data_ptr() or None) if values is not None else None)


def sptir_status_string(status: int) -> str:
    return load_library().sptir_status_string(status).decode()


def sptir_default_bucket_log2(nnz: int, n_rows: int) -> int:
    return int(load_library().sptir_default_bucket_log2(nnz, n_rows))


def sptir_gather_offsets_fit_32(n_cols: int, feat: int) -> bool:
    return bool(load_library().sptir_gather_offsets_fit_32(n_cols, feat))


def sptir_sddmm_default_col_parts(n_rows: int, n_cols: int, nnz: int, feat_hint: int = 0) -> int:
    return int(load_library().sptir_sddmm_default_col_parts(n_rows, n_cols, nnz, feat_hint))


def sptir_launch_plan(n_rows: int, n_cols: int, stored_slots: int, n_col_parts: int, feat: int,
                      options: dict | None = None) -> dict:
    """The launch plan the library would choose for these sizes (host arithmetic only)."""
    out = _LaunchPlan()
    opt = _options(options)
    st = load_library().sptir_launch_plan(n_rows, n_cols, stored_slots, n_col_parts, feat,
                                          ctypes.byref(opt) if opt is not None else None, ctypes.byref(out))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_launch_plan")
    return {name: int(getattr(out, name)) for name, _ in _LaunchPlan._fields_}


class Hyb:
    """Owner of a sptir_hyb_t handle."""

    def __init__(self, handle, n_rows=None, n_cols=None):
        self._h = ctypes.c_void_p(handle)
        self.n_rows, self.n_cols = n_rows, n_cols   # kept here so that sptir_spmm need not ask per call

    @property
    def handle(self):
        if not self._h:
            raise RuntimeError("hyb object already destroyed")
        return self._h

    def destroy(self):
        sptir_hyb_destroy(self)

    def __del__(self):
        try:
            if self._h and _lib is not None:
                _lib.sptir_hyb_destroy(self._h)
                self._h = ctypes.c_void_p(None)
        except Exception:
            pass


def sptir_hyb_build(n_rows: int, n_cols: int, indptr, indices, values, n_col_parts: int,
                    max_bucket_log2: int, stream=None) -> Hyb:
    lib = load_library()
    csr = _csr_struct(n_rows, n_cols, indptr, indices, values)
    out = ctypes.c_void_p(None)
    st = lib.sptir_hyb_build(ctypes.byref(csr), n_col_parts, max_bucket_log2, _stream_ptr(stream), ctypes.byref(out))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_hyb_build")
    return Hyb(out.value, n_rows, n_cols)


def sptir_hyb_build_ex(n_rows: int, n_cols: int, indptr, indices, values, n_col_parts: int,
                       max_bucket_log2: int, options: dict | None = None, stream=None) -> Hyb:
    """sptir_hyb_build with a dict of sptir_build_options_t fields."""
    lib = load_library()
    csr = _csr_struct(n_rows, n_cols, indptr, indices, values)
    out = ctypes.c_void_p(None)
    opt = _options(options)
    st = lib.sptir_hyb_build_ex(ctypes.byref(csr), n_col_parts, max_bucket_log2,
                                ctypes.byref(opt) if opt is not None else None, _stream_ptr(stream), ctypes.byref(out))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_hyb_build_ex")
    return Hyb(out.value, n_rows, n_cols)


def sptir_hyb_search(n_rows: int, n_cols: int, indptr, indices, values, feat: int, c_candidates=(),
                     max_bucket_log2: int = -1, reps: int = 3, stream=None):
    """Builds hyb(c, k) for every candidate c, times SpMM at `feat`, returns (fastest Hyb, its c, [ms per c])."""
    lib = load_library()
    csr = _csr_struct(n_rows, n_cols, indptr, indices, values)
    cands = [int(c) for c in c_candidates]
    n = len(cands)
    arr = (ctypes.c_int32 * max(n, 1))(*cands)
    ms = (ctypes.c_float * max(n, 5))()
    best_c = ctypes.c_int32(0)
    out = ctypes.c_void_p(None)
    st = lib.sptir_hyb_search(ctypes.byref(csr), arr if n else None, n, max_bucket_log2, feat, reps,
                              _stream_ptr(stream), ctypes.byref(out), ctypes.byref(best_c), ms if n else None)
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_hyb_search")
    return Hyb(out.value, n_rows, n_cols), int(best_c.value), [float(ms[i]) for i in range(n)]


def sptir_hyb_destroy(hyb: Hyb) -> None:
    if hyb._h:
        st = load_library().sptir_hyb_destroy(hyb._h)
        hyb._h = ctypes.c_void_p(None)
        if st != SPTIR_OK:
            raise SptirError(st, "sptir_hyb_destroy")


def sptir_hyb_info(hyb: Hyb) -> dict:
    info = _Info()
    st = load_library().sptir_hyb_info(hyb.handle, ctypes.byref(info))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_hyb_info")
    return {name: getattr(info, name) for name, _ in _Info._fields_}


def sptir_hyb_array(hyb: Hyb, name: str) -> np.ndarray:
    """Host copy (numpy) of one canonical hyb array."""
    ptr = ctypes.c_void_p(None)
    n = ctypes.c_int64(0)
    st = load_library().sptir_hyb_array(hyb.handle, ARRAY_IDS[name], ctypes.byref(ptr), ctypes.byref(n))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_hyb_array")
    out = np.empty(n.value, dtype=ARRAY_DTYPES[name])
    if n.value:
        torch.cuda.synchronize()
        rc = _hip_runtime().hipMemcpy(out.ctypes.data, ptr, out.nbytes, 2)  # hipMemcpyDeviceToHost
        if rc != 0:
            raise RuntimeError(f"hipMemcpy failed with {rc}")
    return out


def sptir_spmm(hyb: Hyb, X, Y, stream=None) -> None:
    """Y[n_rows, feat] = A @ X[n_cols, feat]; Y is overwritten."""
    _dev(X, torch.float32, "X"); _dev(Y, torch.float32, "Y")
    if X.dim() != 2 or Y.dim() != 2 or X.shape[1] != Y.shape[1]:
        raise ValueError("X and Y must be 2-D with the same number of columns")
    if X.shape[0] != hyb.n_cols or Y.shape[0] != hyb.n_rows:
        raise ValueError("X / Y row counts do not match the matrix")
    st = load_library().sptir_spmm(hyb.handle, X.data_ptr() or None, Y.data_ptr() or None, X.shape[1],
                                   _stream_ptr(stream))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_spmm")


def sptir_spmm_timed(hyb: Hyb, X, Y, stream=None) -> dict:
    """sptir_spmm with HIP events between its groups of launches; returns their times (ms) and launch counts."""
    _dev(X, torch.float32, "X"); _dev(Y, torch.float32, "Y")
    if X.dim() != 2 or Y.dim() != 2 or X.shape[1] != Y.shape[1]:
        raise ValueError("X and Y must be 2-D with the same number of columns")
    if X.shape[0] != hyb.n_cols or Y.shape[0] != hyb.n_rows:
        raise ValueError("X / Y row counts do not match the matrix")
    out = _SpmmTimes()
    st = load_library().sptir_spmm_timed(hyb.handle, X.data_ptr() or None, Y.data_ptr() or None, X.shape[1],
                                         _stream_ptr(stream), ctypes.byref(out))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_spmm_timed")
    return {name: getattr(out, name) for name, _ in _SpmmTimes._fields_}


def sptir_roof_gather(X, n_rows: int, tiles: int, n_workgroups: int, iters: int, sink, stream=None):
    """(milliseconds, bytes gathered) of one launch of the gather-roof microbenchmark over X[0:n_rows]."""
    _dev(X, torch.float32, "X"); _dev(sink, torch.float32, "sink")
    ms = ctypes.c_float(0.0); nbytes = ctypes.c_double(0.0)
    st = load_library().sptir_roof_gather(X.data_ptr(), n_rows, X.shape[1], tiles, n_workgroups, iters,
                                          sink.data_ptr(), _stream_ptr(stream), ctypes.byref(ms), ctypes.byref(nbytes))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_roof_gather")
    return float(ms.value), float(nbytes.value)


def sptir_roof_fma(n_workgroups: int, iters: int, sink, stream=None):
    """(milliseconds, flops) of one launch of the float32 FMA microbenchmark."""
    _dev(sink, torch.float32, "sink")
    ms = ctypes.c_float(0.0); flops = ctypes.c_double(0.0)
    st = load_library().sptir_roof_fma(n_workgroups, iters, sink.data_ptr(), _stream_ptr(stream), ctypes.byref(ms),
                                       ctypes.byref(flops))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_roof_fma")
    return float(ms.value), float(flops.value)


def sptir_spmm_noalloc(hyb: Hyb, X, Y, stream=None) -> None:
    """sptir_spmm through the entry point that allocates nothing (static scratch inside the library)."""
    _dev(X, torch.float32, "X"); _dev(Y, torch.float32, "Y")
    if X.dim() != 2 or Y.dim() != 2 or X.shape[1] != Y.shape[1]:
        raise ValueError("X and Y must be 2-D with the same number of columns")
    if X.shape[0] != hyb.n_cols or Y.shape[0] != hyb.n_rows:
        raise ValueError("X / Y row counts do not match the matrix")
    st = load_library().sptir_spmm_noalloc(hyb.handle, X.data_ptr() or None, Y.data_ptr() or None, X.shape[1],
                                           _stream_ptr(stream))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_spmm_noalloc")


def sptir_spmm_csr(n_rows: int, n_cols: int, indptr, indices, values, X, Y, stream=None) -> None:
    _dev(X, torch.float32, "X"); _dev(Y, torch.float32, "Y")
    if X.dim() != 2 or Y.dim() != 2 or X.shape[1] != Y.shape[1]:
        raise ValueError("X and Y must be 2-D with the same number of columns")
    if X.shape[0] != n_cols or Y.shape[0] != n_rows:
        raise ValueError("X / Y row counts do not match the matrix")
    csr = _csr_struct(n_rows, n_cols, indptr, indices, values)
    st = load_library().sptir_spmm_csr(ctypes.byref(csr), X.data_ptr() or None, Y.data_ptr() or None, X.shape[1],
                                       _stream_ptr(stream))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_spmm_csr")


# ------------------------------------------------------------ allocator hook
_torch_blocks: dict[int, torch.Tensor] = {}


@_ALLOC_FN
def _torch_alloc(nbytes, ctx, stream):
    # The block is taken from torch's caching allocator under the stream the library will first use it on, so that
    # the allocator orders its reuse (of this block now, and of its memory after the free) against that stream.
    try:
        on = torch.cuda.ExternalStream(int(stream)) if stream else torch.cuda.default_stream()
        with torch.cuda.stream(on):
            t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device="cuda")
    except Exception:
        return None
    _torch_blocks[t.data_ptr()] = t
    return t.data_ptr()


@_FREE_FN
def _torch_free(ptr, ctx):
    _torch_blocks.pop(ptr, None)


def sptir_release_scratch() -> None:
    """Frees the temporary device blocks the library keeps between builds under the default allocator."""
    lib = load_library()
    lib.sptir_release_scratch.restype = ctypes.c_int
    st = lib.sptir_release_scratch()
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_release_scratch")


def sptir_set_allocator(use_torch: bool) -> None:
    """Routes the library's device allocations through torch's caching allocator
    (True) or back to hipMalloc/hipFree (False).  A block belongs to the stream of the call that allocated it
    (the build's stream for a handle's arrays): a handle used on other streams as well must not be destroyed
    while work on them is pending, as with any torch tensor shared between streams."""
    lib = load_library()
    if use_torch:
        st = lib.sptir_set_allocator(_torch_alloc, _torch_free, None)
    else:
        st = lib.sptir_set_allocator(ctypes.cast(None, _ALLOC_FN), ctypes.cast(None, _FREE_FN), None)
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_set_allocator")


def sptir_sddmm_csr(n_rows: int, n_cols: int, indptr, indices, values, X, Yt, B_values, stream=None) -> None:
    """B_values[q] = values[q] * <X[row(q)], Yt[indices[q]]> for every stored position q."""
    _dev(X, torch.float32, "X"); _dev(Yt, torch.float32, "Yt"); _dev(B_values, torch.float32, "B_values")
    if X.dim() != 2 or Yt.dim() != 2 or X.shape[1] != Yt.shape[1]:
        raise ValueError("X and Yt must be 2-D with the same number of columns")
    if X.shape[0] != n_rows or Yt.shape[0] != n_cols:
        raise ValueError("X / Yt row counts do not match the matrix")
    if B_values.dim() != 1 or B_values.shape[0] != values.shape[0]:
        raise ValueError("B_values must have one entry per stored position")
    csr = _csr_struct(n_rows, n_cols, indptr, indices, values)
    st = load_library().sptir_sddmm_csr(ctypes.byref(csr), X.data_ptr() or None, Yt.data_ptr() or None,
                                        B_values.data_ptr() or None, X.shape[1], _stream_ptr(stream))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_sddmm_csr")


class SddmmPlan:
    """Owner of a sptir_sddmm_plan_t handle."""

    def __init__(self, handle, nnz, n_rows, n_cols):
        self._h = ctypes.c_void_p(handle)
        self.nnz, self.n_rows, self.n_cols = nnz, n_rows, n_cols

    @property
    def handle(self):
        if not self._h:
            raise RuntimeError("plan already destroyed")
        return self._h

    def destroy(self):
        sptir_sddmm_plan_destroy(self)

    def __del__(self):
        try:
            if self._h and _lib is not None:
                _lib.sptir_sddmm_plan_destroy(self._h)
                self._h = ctypes.c_void_p(None)
        except Exception:
            pass


def sptir_sddmm_plan_build(n_rows: int, n_cols: int, indptr, indices, n_col_parts: int = 0, feat_hint: int = 0,
                           stream=None) -> SddmmPlan:
    lib = load_library()
    csr = _csr_struct(n_rows, n_cols, indptr, indices, None)
    out = ctypes.c_void_p(None)
    st = lib.sptir_sddmm_plan_build(ctypes.byref(csr), n_col_parts, feat_hint, _stream_ptr(stream), ctypes.byref(out))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_sddmm_plan_build")
    return SddmmPlan(out.value, int(indices.shape[0]), n_rows, n_cols)


def sptir_sddmm(plan: SddmmPlan, values, X, Yt, B_values, stream=None) -> None:
    _dev(values, torch.float32, "values"); _dev(X, torch.float32, "X"); _dev(Yt, torch.float32, "Yt")
    _dev(B_values, torch.float32, "B_values")
    if X.dim() != 2 or Yt.dim() != 2 or X.shape[1] != Yt.shape[1]:
        raise ValueError("X and Yt must be 2-D with the same number of columns")
    if X.shape[0] != plan.n_rows or Yt.shape[0] != plan.n_cols:
        raise ValueError("X / Yt row counts do not match the plan")
    if values.dim() != 1 or values.shape[0] != plan.nnz or B_values.shape != values.shape:
        raise ValueError("values and B_values must have one entry per stored position")
    st = load_library().sptir_sddmm(plan.handle, values.data_ptr() or None, X.data_ptr() or None,
                                    Yt.data_ptr() or None, B_values.data_ptr() or None, X.shape[1],
                                    _stream_ptr(stream))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_sddmm")


def sptir_sddmm_plan_info(plan: SddmmPlan) -> dict:
    info = _PlanInfo()
    st = load_library().sptir_sddmm_plan_info(plan.handle, ctypes.byref(info))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_sddmm_plan_info")
    return {name: getattr(info, name) for name, _ in _PlanInfo._fields_}


def sptir_sddmm_plan_destroy(plan: SddmmPlan) -> None:
    if plan._h:
        st = load_library().sptir_sddmm_plan_destroy(plan._h)
        plan._h = ctypes.c_void_p(None)
        if st != SPTIR_OK:
            raise SptirError(st, "sptir_sddmm_plan_destroy")


class Rgms:
    """Owner of a sptir_rgms_t handle."""

    def __init__(self, handle, n_rel, n_rows, n_cols):
        self._h = ctypes.c_void_p(handle)
        self.n_rel, self.n_rows, self.n_cols = n_rel, n_rows, n_cols

    @property
    def handle(self):
        if not self._h:
            raise RuntimeError("rgms object already destroyed")
        return self._h

    def destroy(self):
        sptir_rgms_destroy(self)

    def __del__(self):
        try:
            if self._h and _lib is not None:
                _lib.sptir_rgms_destroy(self._h)
                self._h = ctypes.c_void_p(None)
        except Exception:
            pass


def sptir_rgms_build(n_relations: int, n_rows: int, n_cols: int, indptr, indices, values, max_bucket_log2: int = -1,
                     workspace_d_out: int = 0, stream=None) -> Rgms:
    """indptr covers the n_relations * n_rows stacked rows (relation after relation)."""
    lib = load_library()
    csr = _csr_struct(n_relations * n_rows, n_cols, indptr, indices, values)
    out = ctypes.c_void_p(None)
    st = lib.sptir_rgms_build(ctypes.byref(csr), n_relations, max_bucket_log2, workspace_d_out, _stream_ptr(stream),
                              ctypes.byref(out))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_rgms_build")
    return Rgms(out.value, n_relations, n_rows, n_cols)


def sptir_rgms(rgms: Rgms, X, W, Y, stream=None) -> None:
    _dev(X, torch.float32, "X"); _dev(W, torch.float32, "W"); _dev(Y, torch.float32, "Y")
    if X.dim() != 2 or W.dim() != 3 or Y.dim() != 2:
        raise ValueError("X and Y must be 2-D, W 3-D")
    if X.shape[0] != rgms.n_cols or Y.shape[0] != rgms.n_rows or W.shape[0] != rgms.n_rel:
        raise ValueError("operand sizes do not match the tensor")
    if W.shape[1] != X.shape[1] or W.shape[2] != Y.shape[1]:
        raise ValueError("W must be [n_relations, d_in, d_out]")
    st = load_library().sptir_rgms(rgms.handle, X.data_ptr() or None, W.data_ptr() or None, Y.data_ptr() or None,
                                   X.shape[1], Y.shape[1], _stream_ptr(stream))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_rgms")


def sptir_rgms_info(rgms: Rgms) -> dict:
    info = _RgmsInfo()
    st = load_library().sptir_rgms_info(rgms.handle, ctypes.byref(info))
    if st != SPTIR_OK:
        raise SptirError(st, "sptir_rgms_info")
    return {name: getattr(info, name) for name, _ in _RgmsInfo._fields_}


def sptir_rgms_destroy(rgms: Rgms) -> None:
    if rgms._h:
        st = load_library().sptir_rgms_destroy(rgms._h)
        rgms._h = ctypes.c_void_p(None)
        if st != SPTIR_OK:
            raise SptirError(st, "sptir_rgms_destroy")
