"""ctypes binding of libtilefusion.so: same entry points as include/tilefusion.h.

Argument marshalling only.  Device operands are passed as objects with a `data_ptr()` method
(torch tensors) or as integer device addresses.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

TF_F32, TF_F64 = 0, 1
TF_FLAG_NO_SPLIT = 1
TF_FLAG_SCHEDULE_ONLY = 2
TF_FLAG_REORDER = 4
TF_FLAG_C_TRANSPOSED = 8
TF_FLAG_SKIP_UNREAD = 16
TF_FLAG_NO_BASELINE = 32

_STATUS = {0: "TF_OK", 1: "TF_EINVAL", 2: "TF_EBADCSR", 3: "TF_ENOMEM", 4: "TF_EHIP",
           5: "TF_EUNSUPPORTED", 6: "TF_EMISMATCH"}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtilefusion.so")
_lib = None


class TfError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status
        self.status_name = _STATUS.get(status, str(status))


class tf_csr(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("n_cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("rowptr", ctypes.c_void_p), ("colidx", ctypes.c_void_p),
                ("vals", ctypes.c_void_p), ("dtype", ctypes.c_int32),
                ("on_device", ctypes.c_int32)]


class tf_tile_params(ctypes.Structure):
    _fields_ = [("ct_size", ctypes.c_int32), ("p", ctypes.c_int32),
                ("fast_mem_bytes", ctypes.c_int64), ("col_slice", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("gather_slices", ctypes.c_int32),
                ("reserved0", ctypes.c_int32)]


class tf_schedule_view(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("nnz", ctypes.c_int64), ("t", ctypes.c_int32),
                ("col_slice", ctypes.c_int32), ("n_slices", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("b_is_sparse", ctypes.c_int32),
                ("reserved0", ctypes.c_int32),
                ("n_coarse_tiles", ctypes.c_int64), ("n_tiles", ctypes.c_int64),
                ("tile_first_ptr", ctypes.POINTER(ctypes.c_int32)),
                ("first_rows", ctypes.POINTER(ctypes.c_int32)),
                ("tile_second_ptr", ctypes.POINTER(ctypes.c_int32)),
                ("second_rows", ctypes.POINTER(ctypes.c_int32)),
                ("n_wf1_units", ctypes.c_int64),
                ("wf1_unit_ptr", ctypes.POINTER(ctypes.c_int32)),
                ("wf1_rows", ctypes.POINTER(ctypes.c_int32)),
                ("spill", ctypes.POINTER(ctypes.c_uint8)),
                ("n_fused_rows", ctypes.c_int64), ("n_wf1_rows", ctypes.c_int64),
                ("n_spill_rows", ctypes.c_int64), ("fused_nnz", ctypes.c_int64),
                ("fused_ratio_eq3", ctypes.c_double), ("fused_ratio_rows", ctypes.c_double),
                ("fused_ratio_nnz", ctypes.c_double),
                ("fast_mem_bytes", ctypes.c_int64), ("lds_fixed_bytes", ctypes.c_int64),
                ("lds_bytes_per_row", ctypes.c_int64), ("lds_row_granule", ctypes.c_int32),
                ("second_block_in_lds", ctypes.c_int32),
                ("eq2_cost_max", ctypes.c_double), ("plan_seconds", ctypes.c_double),
                ("alg_bytes", ctypes.c_int64), ("alg_bytes_unfused", ctypes.c_int64),
                ("second_block_bytes", ctypes.c_int64), ("lds_launch_bytes", ctypes.c_int64),
                ("n_first_rows", ctypes.c_int64),
                ("spill_slot", ctypes.POINTER(ctypes.c_int32)), ("n_direct_rows", ctypes.c_int64),
                ("d1_slices", ctypes.c_int32), ("d1_slice_cols", ctypes.c_int32),
                ("d1_rows", ctypes.c_int64), ("first_wavefront_streams", ctypes.c_int32),
                ("grown_tiles", ctypes.c_int32), ("n_demoted_rows", ctypes.c_int64),
                ("far_rows", ctypes.c_int32), ("automatic", ctypes.c_int32)]


EXPORTS = ["tf_plan_create", "tf_plan_destroy", "tf_plan_schedule", "tf_plan_workspace",
           "tf_gemm_spmm", "tf_gemm_spmm_static", "tf_spmm_spmm", "tf_unfused_gemm_spmm",
           "tf_unfused_spmm_spmm", "tf_run_wavefront", "tf_plan_prepare_unfused", "tf_plan_workspace_unfused",
           "tf_csr_validate", "tf_last_error", "tf_version"]
_INT_RETURNS = [e for e in EXPORTS if e not in ("tf_last_error", "tf_version")]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libtilefusion.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2407_00243_amd.build` "
                          f"(or __graft_entry__.build())")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.tf_plan_create.argtypes = [ctypes.POINTER(tf_csr), i64, i64, i32,
                                   ctypes.POINTER(tf_tile_params), ctypes.POINTER(vp)]
    lib.tf_plan_destroy.argtypes = [vp]
    lib.tf_plan_schedule.argtypes = [vp, ctypes.POINTER(tf_schedule_view)]
    lib.tf_plan_workspace.argtypes = [vp, ctypes.POINTER(vp)]
    lib.tf_gemm_spmm.argtypes = [vp, vp, vp, vp, vp]
    lib.tf_unfused_gemm_spmm.argtypes = [vp, vp, vp, vp, vp]
    lib.tf_gemm_spmm_static.argtypes = [vp, vp, vp, vp, vp]
    lib.tf_spmm_spmm.argtypes = [vp, ctypes.POINTER(tf_csr), vp, vp, vp]
    lib.tf_unfused_spmm_spmm.argtypes = [vp, ctypes.POINTER(tf_csr), vp, vp, vp]
    lib.tf_run_wavefront.argtypes = [vp, i32, vp, ctypes.POINTER(tf_csr), vp, vp, vp]
    lib.tf_plan_prepare_unfused.argtypes = [vp]
    lib.tf_plan_workspace_unfused.argtypes = [vp, ctypes.POINTER(vp)]
    lib.tf_csr_validate.argtypes = [ctypes.POINTER(tf_csr)]
    for name in _INT_RETURNS:
        getattr(lib, name).restype = ctypes.c_int
    lib.tf_last_error.restype = ctypes.c_char_p
    lib.tf_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def tf_last_error() -> str:
    return load_library().tf_last_error().decode()


def tf_version() -> str:
    return load_library().tf_version().decode()


def _check(status: int):
    if status != 0:
        raise TfError(status, tf_last_error())


def _addr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return int(x.data_ptr())


def _dtype_code(dt) -> int:
    s = str(dt)
    if s.endswith("float32"):
        return TF_F32
    if s.endswith("float64"):
        return TF_F64
    raise TypeError(f"unsupported element type {dt}")


class DeviceCsr:
    """A CSR matrix whose three arrays are device tensors (kept alive by this object)."""

    def __init__(self, n_rows: int, n_cols: int, rowptr, colidx, vals):
        self.n_rows, self.n_cols = int(n_rows), int(n_cols)
        self.rowptr, self.colidx, self.vals = rowptr, colidx, vals
        self.nnz = int(colidx.numel())

    def as_struct(self) -> tf_csr:
        return tf_csr(self.n_rows, self.n_cols, self.nnz, _addr(self.rowptr), _addr(self.colidx),
                      _addr(self.vals), _dtype_code(self.vals.dtype), 1)


def _host_csr_struct(A, keep: list) -> tf_csr:
    rowptr = np.ascontiguousarray(A.rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(A.colidx, dtype=np.int32)
    vals = np.ascontiguousarray(A.vals)
    keep.extend([rowptr, colidx, vals])
    return tf_csr(int(A.n_rows), int(A.n_cols), int(colidx.size), rowptr.ctypes.data,
                  colidx.ctypes.data if colidx.size else None,
                  vals.ctypes.data if vals.size else None, _dtype_code(vals.dtype), 0)


def tf_plan_create(A, bcol: int, ccol: int, b_is_sparse: bool, ct_size: int = 0, p: int = 0,
                   fast_mem_bytes: int = 0, col_slice: int = 0, flags: int = 0,
                   gather_slices: int = 0) -> int:
    """A: host CSR (anything with n_rows, n_cols, rowptr, colidx, vals as numpy arrays), a
    DeviceCsr, or a ready tf_csr struct.  Returns the opaque plan handle."""
    lib = load_library()
    keep: list = []
    if isinstance(A, tf_csr):
        a = A
    elif isinstance(A, DeviceCsr):
        a = A.as_struct()
    else:
        a = _host_csr_struct(A, keep)
    tp = tf_tile_params(ct_size, p, fast_mem_bytes, col_slice, flags, gather_slices, 0)
    out = ctypes.c_void_p()
    _check(lib.tf_plan_create(ctypes.byref(a), bcol, ccol, 1 if b_is_sparse else 0,
                              ctypes.byref(tp), ctypes.byref(out)))
    return out.value


def tf_plan_destroy(plan: Optional[int]) -> None:
    _check(load_library().tf_plan_destroy(plan))


def _np_copy(ptr, count: int, dtype) -> np.ndarray:
    if count == 0:
        return np.zeros(0, dtype=dtype)
    return np.ctypeslib.as_array(ptr, shape=(count,)).astype(dtype, copy=True)


def tf_plan_schedule(plan: int) -> dict:
    """Host copy of the plan's schedule: arrays as numpy, counters as Python numbers."""
    v = tf_schedule_view()
    _check(load_library().tf_plan_schedule(plan, ctypes.byref(v)))
    out = {name: getattr(v, name) for name, _ in tf_schedule_view._fields_
           if not name.startswith("reserved")}
    nt, nu = v.n_tiles, v.n_wf1_units
    out["tile_first_ptr"] = _np_copy(v.tile_first_ptr, nt + 1, np.int32)
    out["first_rows"] = _np_copy(v.first_rows, v.n_first_rows, np.int32)
    out["tile_second_ptr"] = _np_copy(v.tile_second_ptr, nt + 1, np.int32)
    out["second_rows"] = _np_copy(v.second_rows, v.n_fused_rows, np.int32)
    out["wf1_unit_ptr"] = _np_copy(v.wf1_unit_ptr, nu + 1, np.int32)
    out["wf1_rows"] = _np_copy(v.wf1_rows, v.n_wf1_rows, np.int32)
    out["spill"] = _np_copy(v.spill, v.n, np.uint8)
    out["spill_slot"] = _np_copy(v.spill_slot, v.n, np.int32)
    return out


def tf_plan_workspace(plan: int) -> int:
    out = ctypes.c_void_p()
    _check(load_library().tf_plan_workspace(plan, ctypes.byref(out)))
    return out.value or 0


def tf_plan_workspace_unfused(plan: int) -> int:
    out = ctypes.c_void_p()
    _check(load_library().tf_plan_workspace_unfused(plan, ctypes.byref(out)))
    return out.value or 0


def tf_plan_prepare_unfused(plan: int) -> None:
    _check(load_library().tf_plan_prepare_unfused(plan))


def tf_csr_validate(M) -> None:
    """M: host CSR (numpy arrays), a DeviceCsr or a tf_csr struct; raises TfError if malformed."""
    keep: list = []
    m = M if isinstance(M, tf_csr) else (M.as_struct() if isinstance(M, DeviceCsr)
                                         else _host_csr_struct(M, keep))
    _check(load_library().tf_csr_validate(ctypes.byref(m)))


def tf_gemm_spmm(plan: int, B, C, D, stream=None) -> None:
    _check(load_library().tf_gemm_spmm(plan, _addr(B), _addr(C), _addr(D), _addr(stream)))


def tf_gemm_spmm_static(plan: int, B, C, D, stream=None) -> None:
    _check(load_library().tf_gemm_spmm_static(plan, _addr(B), _addr(C), _addr(D), _addr(stream)))


def tf_unfused_gemm_spmm(plan: int, B, C, D, stream=None) -> None:
    _check(load_library().tf_unfused_gemm_spmm(plan, _addr(B), _addr(C), _addr(D),
                                               _addr(stream)))


def _csr_arg(B) -> tf_csr:
    return B if isinstance(B, tf_csr) else B.as_struct()


def tf_spmm_spmm(plan: int, B, C, D, stream=None) -> None:
    b = _csr_arg(B)
    _check(load_library().tf_spmm_spmm(plan, ctypes.byref(b), _addr(C), _addr(D), _addr(stream)))


def tf_unfused_spmm_spmm(plan: int, B, C, D, stream=None) -> None:
    b = _csr_arg(B)
    _check(load_library().tf_unfused_spmm_spmm(plan, ctypes.byref(b), _addr(C), _addr(D),
                                               _addr(stream)))


def tf_run_wavefront(plan: int, wavefront: int, B, C, D, stream=None) -> None:
    """B: dense device operand, DeviceCsr / tf_csr, or None (wavefront 1 only)."""
    lib = load_library()
    if B is None or hasattr(B, "data_ptr") or isinstance(B, int):
        _check(lib.tf_run_wavefront(plan, wavefront, _addr(B), None, _addr(C), _addr(D),
                                    _addr(stream)))
    else:
        b = _csr_arg(B)
        _check(lib.tf_run_wavefront(plan, wavefront, None, ctypes.byref(b), _addr(C), _addr(D),
                                    _addr(stream)))


class Plan:
    """Owns a plan handle; a convenience over the tf_* functions."""

    def __init__(self, A, bcol: int, ccol: int, b_is_sparse: bool, **params):
        self.handle = tf_plan_create(A, bcol, ccol, b_is_sparse, **params)
        self.b_is_sparse = bool(b_is_sparse)

    def schedule(self) -> dict:
        return tf_plan_schedule(self.handle)

    def run(self, B, C, D, stream=None) -> None:
        (tf_spmm_spmm if self.b_is_sparse else tf_gemm_spmm)(self.handle, B, C, D, stream)

    def run_unfused(self, B, C, D, stream=None) -> None:
        (tf_unfused_spmm_spmm if self.b_is_sparse else tf_unfused_gemm_spmm)(
            self.handle, B, C, D, stream)

    def run_wavefront(self, wavefront: int, B, C, D, stream=None) -> None:
        tf_run_wavefront(self.handle, wavefront, B, C, D, stream)

    def workspace(self) -> int:
        return tf_plan_workspace(self.handle)

    def workspace_unfused(self) -> int:
        return tf_plan_workspace_unfused(self.handle)

    def prepare_unfused(self) -> None:
        tf_plan_prepare_unfused(self.handle)

    def close(self) -> None:
        if self.handle:
            tf_plan_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
