"""CPU oracle for the preprocessing of the paper's sparse-matrix evaluation -- TEST INFRASTRUCTURE ONLY.

The evaluation section (IV-A, "Baselines and datasets") reorders every matrix with the Reverse
Cuthill-McKee algorithm of scipy before building the formats, and reads its matrices from Matrix Market
files.  Here these steps are the library routines themselves (scipy) plus plain numpy definitions; the GPU
library's own C++ versions are compared against them.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this module; it never imports the GPU library.
"""
from __future__ import annotations

import numpy as np
import scipy.io
import scipy.sparse as sp
from scipy.sparse.csgraph import reverse_cuthill_mckee


def _pattern(m, k, row_ptr, col_idx):
    rp = np.asarray(row_ptr, dtype=np.int64)
    ci = np.asarray(col_idx, dtype=np.int64)
    return sp.csr_matrix((np.ones(len(ci), dtype=np.int8), ci, rp), shape=(m, k))


def rcm(m, row_ptr, col_idx) -> np.ndarray:
    """Reverse Cuthill-McKee permutation of a square matrix's structure, taken as A + A^T (Section IV-A).

    perm[new] = old, int32.  This is scipy's routine, the one the paper names.
    """
    return np.asarray(reverse_cuthill_mckee(_pattern(m, m, row_ptr, col_idx), symmetric_mode=False), dtype=np.int32)


def sym_adjacency(m, row_ptr, col_idx):
    """Neighbour lists of the structure of A + A^T (a stored diagonal entry makes a node its own neighbour)."""
    a = _pattern(m, m, row_ptr, col_idx)
    s = (a + a.T).tocsr()
    s.sort_indices()
    return s.indptr.astype(np.int64), s.indices.astype(np.int64)


def degrees(m, row_ptr, col_idx) -> np.ndarray:
    """The key by which Cuthill-McKee orders nodes: neighbours in A + A^T, a stored diagonal entry counting twice
    (scipy's convention: the self-loop is a neighbour and is then counted once more)."""
    indptr, indices = sym_adjacency(m, row_ptr, col_idx)
    deg = np.diff(indptr)
    rows = np.repeat(np.arange(m, dtype=np.int64), deg)
    return deg + np.bincount(rows[indices == rows], minlength=m)


def bandwidth(m, row_ptr, col_idx) -> int:
    """max |i - j| over stored entries (0 for an empty matrix)."""
    rp = np.asarray(row_ptr, dtype=np.int64)
    ci = np.asarray(col_idx, dtype=np.int64)
    if len(ci) == 0:
        return 0
    rows = np.repeat(np.arange(m, dtype=np.int64), np.diff(rp))
    return int(np.abs(rows - ci).max())


def permute_csr(m, k, row_ptr, col_idx, values, row_perm, col_perm=None):
    """A'[i][j] = A[row_perm[i]][col_perm[j]] as sorted CSR; col_perm None keeps the columns.

    Returns (row_ptr int32, col_idx int32, values of the input dtype).  Values are copied, never changed.
    """
    rp = np.asarray(row_ptr, dtype=np.int64)
    ci = np.asarray(col_idx, dtype=np.int64)
    va = np.asarray(values)
    row_perm = np.asarray(row_perm, dtype=np.int64)
    new_col_of = np.arange(k, dtype=np.int64)
    if col_perm is not None:
        new_col_of = np.empty(k, dtype=np.int64)
        new_col_of[np.asarray(col_perm, dtype=np.int64)] = np.arange(k, dtype=np.int64)
    out_rp = np.zeros(m + 1, dtype=np.int64)
    out_ci, out_va = [], []
    for i in range(m):
        old = row_perm[i]
        cols = new_col_of[ci[rp[old]:rp[old + 1]]]
        vals = va[rp[old]:rp[old + 1]]
        order = np.argsort(cols, kind="stable")
        out_ci.append(cols[order])
        out_va.append(vals[order])
        out_rp[i + 1] = out_rp[i] + len(cols)
    cat_ci = np.concatenate(out_ci) if out_ci else np.zeros(0, np.int64)
    cat_va = np.concatenate(out_va) if out_va else va[:0]
    return out_rp.astype(np.int32), cat_ci.astype(np.int32), cat_va.astype(va.dtype)


def read_mtx(path):
    """Matrix Market coordinate file -> (m, k, row_ptr, col_idx, values float32), sorted CSR.

    scipy's reader expands symmetric / skew-symmetric storage; duplicates are summed (in float64), explicit zeros
    are kept, pattern files get the value 1.
    """
    a = scipy.io.mmread(path)
    a = sp.coo_matrix(a).astype(np.float64).tocsr()
    a.sum_duplicates()
    a.sort_indices()
    return (a.shape[0], a.shape[1], a.indptr.astype(np.int32), a.indices.astype(np.int32),
            a.data.astype(np.float32))
