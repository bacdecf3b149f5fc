"""ctypes binding of libasyncsparse.so: same names as the C ABI, argument marshalling only.

Every step of the path (format conversion, task partition, the SpMM kernels) runs inside the
library; nothing here computes.  Loading fails loudly when the library has not been built
(``python -m paper_2604_17834_amd.build``) -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# ASP_LIBRARY names another build of the same library (the host-sanitized one of the CPU-only tests)
LIB_PATH = os.environ.get("ASP_LIBRARY") or os.path.join(_PKG, "libasyncsparse.so")

ASP_OK = 0
ASP_ERR_INVALID_ARG, ASP_ERR_INVALID_CSR, ASP_ERR_UNSUPPORTED = 1, 2, 3
ASP_ERR_OUT_OF_MEMORY, ASP_ERR_HIP, ASP_ERR_BUFFER_TOO_SMALL = 4, 5, 6
ASP_FMT_BCSR, ASP_FMT_WCSR = 0, 1
ASP_DT_BF16, ASP_DT_F32 = 0, 1
ASP_ARR_ROW_PTR, ASP_ARR_COL_IDX, ASP_ARR_VALUES, ASP_ARR_TASKS = 0, 1, 2, 3
ASP_FLAG_HOST_CONVERT_ONLY = 1
ASP_MAX_N = 65535 * 64   # largest dense width any call accepts

_FMT = {"bcsr": ASP_FMT_BCSR, "wcsr": ASP_FMT_WCSR}
_DT = {"bf16": ASP_DT_BF16, "f32": ASP_DT_F32}
_NP = {ASP_DT_BF16: np.uint16, ASP_DT_F32: np.float32}

EXPORTED_SYMBOLS = [
    "asp_create_from_csr", "asp_spmm", "asp_spmm_static_scratch", "asp_spmm_xt", "asp_reserve", "asp_rcm", "asp_permute_csr",
    "asp_mtx_read", "asp_mtx_get", "asp_mtx_free", "asp_get_info", "asp_plan_spmm", "asp_export", "asp_destroy",
    "asp_status_string", "asp_last_error",
]


class asp_config_t(ctypes.Structure):
    _fields_ = [("format", ctypes.c_int32), ("dtype", ctypes.c_int32), ("b_row", ctypes.c_int32),
                ("b_col", ctypes.c_int32), ("task_cols", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class asp_info_t(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("k", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("format", ctypes.c_int32), ("dtype", ctypes.c_int32), ("b_row", ctypes.c_int32),
                ("b_col", ctypes.c_int32), ("task_cols", ctypes.c_int32), ("on_device", ctypes.c_int32),
                ("n_brows", ctypes.c_int64), ("n_units", ctypes.c_int64), ("n_tasks", ctypes.c_int64),
                ("n_zero_rows_units", ctypes.c_int64), ("fill_ratio", ctypes.c_double)]


class asp_plan_t(ctypes.Structure):
    _fields_ = [("bn", ctypes.c_int32), ("n_tiles", ctypes.c_int32), ("vectorized", ctypes.c_int32),
                ("workgroups", ctypes.c_int64), ("padded_n", ctypes.c_int64)]


class AspError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        L = lib()
        name = L.asp_status_string(status).decode()
        detail = L.asp_last_error().decode()
        super().__init__("%s: %s (%s)" % (where, name, detail))


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libasyncsparse.so is missing: build it with `python -m paper_2604_17834_amd.build` "
                           "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    L.asp_create_from_csr.argtypes = [ctypes.POINTER(asp_config_t), i64, i64, i64, vp, vp, vp, vp,
                                      ctypes.POINTER(vp)]
    L.asp_create_from_csr.restype = ctypes.c_int
    L.asp_spmm.argtypes = [vp, vp, vp, i64, vp]
    L.asp_spmm.restype = ctypes.c_int
    L.asp_spmm_static_scratch.argtypes = [vp, vp, vp, i64, vp]
    L.asp_spmm_static_scratch.restype = ctypes.c_int
    L.asp_spmm_xt.argtypes = [vp, vp, vp, i64, vp]
    L.asp_spmm_xt.restype = ctypes.c_int
    L.asp_reserve.argtypes = [vp, i64]
    L.asp_reserve.restype = ctypes.c_int
    L.asp_rcm.argtypes = [i64, vp, vp, vp]
    L.asp_rcm.restype = ctypes.c_int
    L.asp_permute_csr.argtypes = [i64, i64, vp, vp, vp, ctypes.c_int32, vp, vp, vp, vp, vp]
    L.asp_permute_csr.restype = ctypes.c_int
    L.asp_mtx_read.argtypes = [ctypes.c_char_p, ctypes.POINTER(vp)]
    L.asp_mtx_read.restype = ctypes.c_int
    L.asp_mtx_get.argtypes = [vp] + [ctypes.POINTER(i64)] * 3 + [ctypes.POINTER(vp)] * 3
    L.asp_mtx_get.restype = ctypes.c_int
    L.asp_mtx_free.argtypes = [vp]
    L.asp_mtx_free.restype = ctypes.c_int
    L.asp_get_info.argtypes = [vp, ctypes.POINTER(asp_info_t)]
    L.asp_get_info.restype = ctypes.c_int
    L.asp_plan_spmm.argtypes = [vp, i64, ctypes.POINTER(asp_plan_t)]
    L.asp_plan_spmm.restype = ctypes.c_int
    L.asp_export.argtypes = [vp, ctypes.c_int, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
    L.asp_export.restype = ctypes.c_int
    L.asp_destroy.argtypes = [vp]
    L.asp_destroy.restype = ctypes.c_int
    L.asp_status_string.argtypes = [ctypes.c_int]
    L.asp_status_string.restype = ctypes.c_char_p
    L.asp_last_error.argtypes = []
    L.asp_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _ptr(a):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.c_void_p)


def asp_create_from_csr(fmt, dtype, b_row, b_col, m, k, row_ptr, col_idx, values, task_cols=0, flags=0,
                        stream=None, check=True):
    """Returns an opaque handle (int).  CSR arrays are numpy host arrays; they are passed as they are
    (int32 indices, uint16/float32 values) -- wrong dtypes are converted here, nothing else."""
    L = lib()
    cfg = asp_config_t(_FMT.get(fmt, fmt), _DT.get(dtype, dtype), b_row, b_col, task_cols, flags)
    rp = None if row_ptr is None else np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = None if col_idx is None else np.ascontiguousarray(col_idx, dtype=np.int32)
    va = None if values is None else np.ascontiguousarray(values, dtype=_NP.get(cfg.dtype, np.float32))
    nnz = 0 if ci is None else len(ci)
    out = ctypes.c_void_p()
    st = L.asp_create_from_csr(ctypes.byref(cfg), m, k, nnz, _ptr(rp), _ptr(ci), _ptr(va), stream,
                               ctypes.byref(out))
    if check and st != ASP_OK:
        raise AspError(st, "asp_create_from_csr")
    return out.value if check else (st, out.value)


def asp_spmm(handle, B_ptr, C_ptr, N, stream=None, check=True):
    """B_ptr / C_ptr are device addresses (e.g. torch tensor .data_ptr()), stream a hipStream_t value."""
    st = lib().asp_spmm(handle, B_ptr, C_ptr, N, stream)
    if check and st != ASP_OK:
        raise AspError(st, "asp_spmm")
    return st


ASP_STATIC_SCRATCH_BYTES = 64 << 20


def asp_spmm_static_scratch(handle, B_ptr, C_ptr, N, stream=None, check=True):
    """asp_spmm for callers that cannot allocate: split WCSR windows use the library's static scratch array."""
    st = lib().asp_spmm_static_scratch(handle, B_ptr, C_ptr, N, stream)
    if check and st != ASP_OK:
        raise AspError(st, "asp_spmm_static_scratch")
    return st


def asp_reserve(handle, N, check=True):
    """Scratch memory for asp_spmm calls of width up to N (only bf16 WCSR handles with split windows need any)."""
    st = lib().asp_reserve(handle, N)
    if check and st != ASP_OK:
        raise AspError(st, "asp_reserve")
    return st


def asp_rcm(m, row_ptr, col_idx) -> np.ndarray:
    """Reverse Cuthill-McKee permutation (perm[new] = old) of a square CSR structure; host only."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    perm = np.empty(m, dtype=np.int32)
    st = lib().asp_rcm(m, rp.ctypes.data, ci.ctypes.data if len(ci) else None, perm.ctypes.data)
    if st != ASP_OK:
        raise AspError(st, "asp_rcm")
    return perm


def asp_permute_csr(m, k, row_ptr, col_idx, values, dtype, row_perm, col_perm=None, check=True):
    """A'[i][j] = A[row_perm[i]][col_perm[j]]; returns (row_ptr, col_idx, values) or the status when check is False."""
    dt = _DT.get(dtype, dtype)
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    va = np.ascontiguousarray(values, dtype=_NP[dt])
    rperm = np.ascontiguousarray(row_perm, dtype=np.int32)
    cperm = None if col_perm is None else np.ascontiguousarray(col_perm, dtype=np.int32)
    orp, oci, ova = np.empty(m + 1, np.int32), np.empty(len(ci), np.int32), np.empty(len(va), _NP[dt])
    st = lib().asp_permute_csr(m, k, rp.ctypes.data, ci.ctypes.data if len(ci) else None,
                               va.ctypes.data if len(va) else None, dt, rperm.ctypes.data,
                               None if cperm is None else cperm.ctypes.data, orp.ctypes.data,
                               oci.ctypes.data if len(oci) else None, ova.ctypes.data if len(ova) else None)
    if st != ASP_OK:
        if check:
            raise AspError(st, "asp_permute_csr")
        return st
    return orp, oci, ova


def asp_mtx_read(path, check=True):
    """Matrix Market coordinate file -> (m, k, row_ptr, col_idx, values float32) as numpy copies; host only."""
    h = ctypes.c_void_p()
    st = lib().asp_mtx_read(os.fsencode(path), ctypes.byref(h))
    if st != ASP_OK:
        if check:
            raise AspError(st, "asp_mtx_read")
        return st
    try:
        m, k, nnz = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        prp, pci, pva = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        st = lib().asp_mtx_get(h, ctypes.byref(m), ctypes.byref(k), ctypes.byref(nnz), ctypes.byref(prp),
                               ctypes.byref(pci), ctypes.byref(pva))
        if st != ASP_OK:
            raise AspError(st, "asp_mtx_get")

        def copy(ptr, n, ct, dt):
            if n == 0:
                return np.zeros(0, dt)
            return np.ctypeslib.as_array(ctypes.cast(ptr, ctypes.POINTER(ct)), shape=(n,)).astype(dt, copy=True)
        return (m.value, k.value, copy(prp, m.value + 1, ctypes.c_int32, np.int32),
                copy(pci, nnz.value, ctypes.c_int32, np.int32), copy(pva, nnz.value, ctypes.c_float, np.float32))
    finally:
        lib().asp_mtx_free(h)


def asp_spmm_xt(handle, X_ptr, Y_ptr, N, stream=None, check=True):
    """Y[N x m] = X[N x k] x A^T; X_ptr / Y_ptr are device addresses, stream a hipStream_t value."""
    st = lib().asp_spmm_xt(handle, X_ptr, Y_ptr, N, stream)
    if check and st != ASP_OK:
        raise AspError(st, "asp_spmm_xt")
    return st


def asp_get_info(handle) -> asp_info_t:
    info = asp_info_t()
    st = lib().asp_get_info(handle, ctypes.byref(info))
    if st != ASP_OK:
        raise AspError(st, "asp_get_info")
    return info


def asp_plan_spmm(handle, N) -> asp_plan_t:
    plan = asp_plan_t()
    st = lib().asp_plan_spmm(handle, N, ctypes.byref(plan))
    if st != ASP_OK:
        raise AspError(st, "asp_plan_spmm")
    return plan


def asp_export(handle, which) -> np.ndarray:
    """Canonical array as numpy, shaped as the header documents."""
    L = lib()
    info = asp_get_info(handle)
    need = ctypes.c_size_t()
    st = L.asp_export(handle, which, None, 0, ctypes.byref(need))
    if st not in (ASP_OK, ASP_ERR_BUFFER_TOO_SMALL):
        raise AspError(st, "asp_export(query)")
    dt = _NP[info.dtype] if which == ASP_ARR_VALUES else np.int32
    out = np.empty(need.value // np.dtype(dt).itemsize, dtype=dt)
    if need.value:
        st = L.asp_export(handle, which, _ptr(out), need.value, None)
        if st != ASP_OK:
            raise AspError(st, "asp_export")
    if which == ASP_ARR_VALUES:
        if info.format == ASP_FMT_BCSR:
            return out.reshape(info.n_units, info.b_row, info.b_col)
        return out.reshape(info.n_units // info.b_col, info.b_row, info.b_col)
    if which == ASP_ARR_TASKS:
        return out.reshape(-1, 4)
    return out


def asp_destroy(handle):
    if handle:
        lib().asp_destroy(handle)


def asp_status_string(status: int) -> str:
    return lib().asp_status_string(status).decode()


def asp_last_error() -> str:
    return lib().asp_last_error().decode()
