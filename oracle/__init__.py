"""CPU oracle for BCSR / WCSR SpMM -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end of ``asp_oracle.c`` (plain C, fp64 accumulation).  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library never does, and this package never imports the GPU
library.  It follows the paper's Section II-C (problem statement and the two
formats), Section III-C (sub-tasks of long row-windows) and Section IV-C
(tile-width rule).

dtype strings: "bf16" (uint16 bit patterns) or "f32".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asp_oracle.c")
_LIB = os.path.join(_HERE, "libasp_oracle.so")
_lib = None

_DT = {"bf16": 0, "f32": 1}
_NP = {"bf16": np.uint16, "f32": np.float32}


# ASP_ORACLE_SANITIZE=1: the same source under AddressSanitizer + UndefinedBehaviorSanitizer (clang, so that its
# runtime is the one the host-sanitized build of the library uses); the process must preload that runtime
_SANITIZE = os.environ.get("ASP_ORACLE_SANITIZE") == "1"
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libasp_oracle_hostsan.so")
_CLANG = "/opt/rocm/lib/llvm/bin/clang"


def build(force: bool = False) -> str:
    """Compile asp_oracle.c with gcc (OpenMP) into oracle/libasp_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        if _SANITIZE:
            subprocess.check_call([_CLANG, "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                                   "-fno-sanitize-recover=undefined", "-shared-libsan", "-fopenmp", "-shared", "-fPIC",
                                   "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
        else:
            subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                                   "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    i64, i32, vp, dbl = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_double
    L.oracle_num_threads.restype = ctypes.c_int
    L.oracle_spmm.argtypes = [i64, i64, vp, vp, vp, ctypes.c_int, vp, i64, i64, vp, vp]
    L.oracle_spmm.restype = ctypes.c_int
    L.oracle_bcsr_count.argtypes = [i64, i64, vp, vp, i32, i32, vp]
    L.oracle_bcsr_count.restype = i64
    L.oracle_bcsr_fill.argtypes = [i64, i64, vp, vp, vp, ctypes.c_int, i32, i32, vp, vp, vp]
    L.oracle_bcsr_fill.restype = ctypes.c_int
    L.oracle_fill_ratio.argtypes = [i64, i64, i32, i32]
    L.oracle_fill_ratio.restype = dbl
    L.oracle_wcsr_count.argtypes = [i64, i64, vp, vp, i32, i32, vp]
    L.oracle_wcsr_count.restype = i64
    L.oracle_wcsr_fill.argtypes = [i64, i64, vp, vp, vp, ctypes.c_int, i32, i32, vp, vp, vp]
    L.oracle_wcsr_fill.restype = ctypes.c_int
    L.oracle_wcsr_tasks.argtypes = [i64, vp, i32, vp]
    L.oracle_wcsr_tasks.restype = i64
    L.oracle_padded_width.argtypes = [i64, i64]
    L.oracle_padded_width.restype = i64
    L.oracle_choose_bn.argtypes = [i64, vp, ctypes.c_int]
    L.oracle_choose_bn.restype = i64
    L.oracle_choose_bn_weighted.argtypes = [i64, vp, vp, ctypes.c_int]
    L.oracle_choose_bn_weighted.restype = i64
    L.oracle_choose_bn_filled.argtypes = [i64, vp, vp, ctypes.c_int, i64, i64]
    L.oracle_choose_bn_filled.restype = i64
    _lib = L
    return L


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _csr_args(row_ptr, col_idx, values, dtype):
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    va = np.ascontiguousarray(values, dtype=_NP[dtype])
    assert rp[0] == 0 and len(ci) == rp[-1] == len(va)
    return rp, ci, va


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def spmm(m, k, row_ptr, col_idx, values, dtype, B, want_bound=True):
    """C = A x B in fp64 (Section II-C) and S = |A| x |B|.  B: [k, N] array of the same dtype.

    Returns (C, S) as float64 [m, N]; S is None when want_bound is False.
    """
    L = _load()
    rp, ci, va = _csr_args(row_ptr, col_idx, values, dtype)
    Bc = np.ascontiguousarray(B, dtype=_NP[dtype])
    assert Bc.ndim == 2 and Bc.shape[0] == k and len(rp) == m + 1
    N = Bc.shape[1]
    C = np.empty((m, N), dtype=np.float64)
    S = np.empty((m, N), dtype=np.float64) if want_bound else None
    rc = L.oracle_spmm(m, k, _p(rp), _p(ci), _p(va), _DT[dtype], _p(Bc), N, N, _p(C),
                       _p(S) if want_bound else None)
    assert rc == 0
    return C, S


def to_bcsr(m, k, row_ptr, col_idx, values, dtype, b_row, b_col):
    """CSR -> BCSR (Section II-C).  Returns (block_row_ptr, block_col_idx, blocks[nnzb, b_row, b_col])."""
    L = _load()
    rp, ci, va = _csr_args(row_ptr, col_idx, values, dtype)
    nbr = -(-m // b_row)
    brp = np.zeros(nbr + 1, dtype=np.int32)
    nb = L.oracle_bcsr_count(m, k, _p(rp), _p(ci), b_row, b_col, _p(brp))
    bci = np.zeros(nb, dtype=np.int32)
    blocks = np.zeros((nb, b_row, b_col), dtype=_NP[dtype])
    L.oracle_bcsr_fill(m, k, _p(rp), _p(ci), _p(va), _DT[dtype], b_row, b_col, _p(brp), _p(bci), _p(blocks))
    return brp, bci, blocks


def fill_ratio(nnz, nnz_blocks, b_row, b_col) -> float:
    return float(_load().oracle_fill_ratio(nnz, nnz_blocks, b_row, b_col))


def to_wcsr(m, k, row_ptr, col_idx, values, dtype, b_row, b_col):
    """CSR -> WCSR (Section II-C).

    Returns (window_row_ptr, window_col_idx, values[padded/b_col, b_row, b_col]).
    """
    L = _load()
    rp, ci, va = _csr_args(row_ptr, col_idx, values, dtype)
    nw = -(-m // b_row)
    wrp = np.zeros(nw + 1, dtype=np.int32)
    padded = L.oracle_wcsr_count(m, k, _p(rp), _p(ci), b_row, b_col, _p(wrp))
    wci = np.zeros(padded, dtype=np.int32)
    vals = np.zeros((padded // b_col, b_row, b_col), dtype=_NP[dtype])
    L.oracle_wcsr_fill(m, k, _p(rp), _p(ci), _p(va), _DT[dtype], b_row, b_col, _p(wrp), _p(wci), _p(vals))
    return wrp, wci, vals


def wcsr_tasks(window_row_ptr, task_cols):
    """Sub-tasks of row-windows (Section III-C).  Returns int32 [n_tasks, 4]."""
    L = _load()
    wrp = np.ascontiguousarray(window_row_ptr, dtype=np.int32)
    nw = len(wrp) - 1
    nt = L.oracle_wcsr_tasks(nw, _p(wrp), task_cols, None)
    tasks = np.zeros((nt, 4), dtype=np.int32)
    if nt:
        L.oracle_wcsr_tasks(nw, _p(wrp), task_cols, _p(tasks))
    return tasks


def padded_width(N, BN) -> int:
    return int(_load().oracle_padded_width(N, BN))


def choose_bn(N, candidates) -> int:
    c = np.ascontiguousarray(candidates, dtype=np.int64)
    return int(_load().oracle_choose_bn(N, _p(c), len(c)))


def choose_bn_weighted(N, candidates, cost) -> int:
    """Tile width with the least padded_width x cost per column (Section IV-C); ties: the larger."""
    c = np.ascontiguousarray(candidates, dtype=np.int64)
    w = np.ascontiguousarray(cost, dtype=np.int64)
    assert len(c) == len(w)
    return int(_load().oracle_choose_bn_weighted(N, _p(c), _p(w), len(c)))


def choose_bn_filled(N, candidates, cost, rows, units) -> int:
    """choose_bn_weighted, then the next narrower candidate while rows x ceil(N / BN) tiles are fewer than `units`."""
    c = np.ascontiguousarray(candidates, dtype=np.int64)
    w = np.ascontiguousarray(cost, dtype=np.int64)
    assert len(c) == len(w)
    return int(_load().oracle_choose_bn_filled(N, _p(c), _p(w), len(c), rows, units))
