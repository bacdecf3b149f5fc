"""Seeded synthetic inputs for the SpMM path: sparse A in CSR, dense B.

This module only draws inputs.  It holds none of the method's arithmetic (no
format conversion, no products) so that the CPU oracle and the HIP library can
both be fed from it without sharing anything that is under test.

All sparse matrices come back as a :class:`Csr` (int32 ``row_ptr``/``col_idx``,
column indices strictly ascending inside a row).  bf16 data is carried as
``uint16`` bit patterns, fp32 data as ``float32``.

The workloads stand in for the paper's inputs: randomly block-sparsified FFN
weights (LLM case study, Section IV-D) and irregular SuiteSparse-like matrices
(Section IV-A), neither of which is available offline.
"""
from __future__ import annotations

import re
from dataclasses import dataclass

import numpy as np

BF16 = "bf16"
F32 = "f32"


@dataclass
class Csr:
    m: int
    k: int
    row_ptr: np.ndarray  # int32 [m+1]
    col_idx: np.ndarray  # int32 [nnz]
    values: np.ndarray   # uint16 (bf16 bits) or float32 [nnz]
    dtype: str           # BF16 or F32

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (storage format of the inputs, not arithmetic)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == BF16:
        return f32_to_bf16_bits(x)
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored data to float64 (for test-side bookkeeping)."""
    if dtype == BF16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


# --------------------------------------------------------------------------
# dense operands
# --------------------------------------------------------------------------
def dense_normal(rows: int, cols: int, dtype: str, seed: int, std: float = 1.0) -> np.ndarray:
    """Row-major rows x cols matrix of N(0, std^2) samples."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return _store(x, dtype)


def dense_identity(k: int, dtype: str) -> np.ndarray:
    return _store(np.eye(k, dtype=np.float32), dtype)


# --------------------------------------------------------------------------
# CSR assembly from (row, col) keys
# --------------------------------------------------------------------------
def _csr_from_keys(m: int, k: int, keys: np.ndarray, values_fn, dtype: str) -> Csr:
    """keys = row * k + col (int64), need not be unique or sorted."""
    keys = np.unique(keys)  # sorted ascending, deduped
    rows = keys // k
    cols = (keys - rows * k).astype(np.int32)
    counts = np.bincount(rows, minlength=m)
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    assert row_ptr[-1] < 2**31
    vals = values_fn(len(keys))
    return Csr(m, k, row_ptr.astype(np.int32), cols, _store(vals, dtype), dtype)


def random_csr(m: int, k: int, density: float, seed: int, dtype: str = F32,
               empty_row_frac: float = 0.0, dist: str = "uniform") -> Csr:
    """Small unstructured matrix for tests: each entry kept with prob. density."""
    rng = np.random.default_rng(seed)
    mask = rng.random((m, k)) < density
    if empty_row_frac > 0:
        mask[rng.random(m) < empty_row_frac, :] = False
    rows, cols = np.nonzero(mask)
    keys = rows.astype(np.int64) * k + cols

    def vals(n):
        if dist == "uniform":
            return rng.uniform(-1.0, 1.0, n).astype(np.float32)
        return (rng.standard_normal(n) * 0.02).astype(np.float32)

    return _csr_from_keys(m, k, keys, vals, dtype)


# --------------------------------------------------------------------------
# block-sparse weights (stand-in for block-pruned FFN projections)
# --------------------------------------------------------------------------
def _csr_from_block_mask(m: int, k: int, b_row: int, b_col: int, mask: np.ndarray,
                         rng: np.random.Generator, std: float, dtype: str) -> Csr:
    """Every element of a kept block is a stored entry with an N(0,std^2) value."""
    nbr, nbc = mask.shape
    # widths of block columns / heights of block rows (ragged last ones)
    col_w = np.minimum(b_col, k - np.arange(nbc) * b_col)
    row_h = np.minimum(b_row, m - np.arange(nbr) * b_row)
    per_brow_cols = (mask * col_w[None, :]).sum(axis=1)          # entries per row in block-row
    row_len = np.repeat(per_brow_cols, row_h)                     # [m]
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(row_len, out=row_ptr[1:])
    nnz = int(row_ptr[-1])
    assert nnz < 2**31
    col_idx = np.empty(nnz, dtype=np.int32)
    for I in range(nbr):
        js = np.nonzero(mask[I])[0]
        if len(js) == 0:
            continue
        cols = np.concatenate([np.arange(J * b_col, J * b_col + col_w[J], dtype=np.int32) for J in js])
        r0 = I * b_row
        seg = col_idx[row_ptr[r0]:row_ptr[r0 + row_h[I]]]
        seg.reshape(row_h[I], len(cols))[:] = cols[None, :]
    vals = rng.standard_normal(nnz, dtype=np.float32) * np.float32(std)
    return Csr(m, k, row_ptr.astype(np.int32), col_idx, _store(vals, dtype), dtype)


def block_sparse_bernoulli(m: int, k: int, b_row: int, b_col: int, sparsity: float, seed: int,
                           dtype: str = BF16, std: float = 0.02) -> Csr:
    """Uniform-random block mask: each block kept with probability 1 - sparsity."""
    rng = np.random.default_rng(seed)
    nbr, nbc = -(-m // b_row), -(-k // b_col)
    mask = rng.random((nbr, nbc)) >= sparsity
    return _csr_from_block_mask(m, k, b_row, b_col, mask, rng, std, dtype)


def block_sparse_geometric(m: int, k: int, b_row: int, b_col: int, sparsity: float, seed: int,
                           dtype: str = BF16, std: float = 0.02) -> Csr:
    """Block mask with geometric per-block-row lengths (load-imbalance variant).

    Block-row I keeps L_I = min(nbc, G) distinct uniform block columns, G
    geometric on {0,1,...} with mean (1 - sparsity) * nbc.
    """
    rng = np.random.default_rng(seed)
    nbr, nbc = -(-m // b_row), -(-k // b_col)
    mu = (1.0 - sparsity) * nbc
    p = 1.0 / (1.0 + mu)
    L = np.minimum(nbc, rng.geometric(p, nbr) - 1)
    mask = np.zeros((nbr, nbc), dtype=bool)
    for I in range(nbr):
        if L[I] > 0:
            mask[I, rng.choice(nbc, size=int(L[I]), replace=False)] = True
    return _csr_from_block_mask(m, k, b_row, b_col, mask, rng, std, dtype)


# --------------------------------------------------------------------------
# irregular graph-like matrices (stand-in for SuiteSparse inputs)
# --------------------------------------------------------------------------
def zipf_graph(m: int, k: int, target_nnz: int, seed: int, alpha: float = 2.0, cap: int = 50000,
               dtype: str = F32) -> Csr:
    """Row lengths ~ Zipf(alpha) rescaled to hit target_nnz, capped; uniform columns; U(-1,1) values."""
    rng = np.random.default_rng(seed)
    raw = rng.zipf(alpha, m).astype(np.float64)
    raw = np.minimum(raw, 1e9)
    cap = min(cap, k)
    f = target_nnz / raw.sum()
    for _ in range(8):  # capping loses mass; rescale a few times so the total lands near target
        lens = np.minimum(cap, np.maximum(1, np.rint(f * raw))).astype(np.int64)
        f *= target_nnz / lens.sum()
    rows = np.repeat(np.arange(m, dtype=np.int64), lens)
    cols = rng.integers(0, k, size=rows.shape[0], dtype=np.int64)
    keys = rows * k + cols
    del rows, cols
    return _csr_from_keys(m, k, keys, lambda n: rng.uniform(-1.0, 1.0, n).astype(np.float32), dtype)


def banded_plus_dense_rows(m: int, seed: int, half_band: int = 13, n_dense_rows: int = 64,
                           dense_row_nnz: int = 200000, dtype: str = F32) -> Csr:
    """Square matrix: band of 2*half_band+1 diagonals plus a few very long rows (random columns)."""
    rng = np.random.default_rng(seed)
    k = m
    i = np.arange(m, dtype=np.int64)
    parts = []
    for d in range(-half_band, half_band + 1):
        j = i + d
        ok = (j >= 0) & (j < k)
        parts.append(i[ok] * k + j[ok])
    n_dense_rows = min(n_dense_rows, m)
    dense_rows = rng.choice(m, size=n_dense_rows, replace=False).astype(np.int64)
    dense_row_nnz = min(dense_row_nnz, k)
    for r in dense_rows:
        parts.append(r * k + rng.integers(0, k, size=dense_row_nnz, dtype=np.int64))
    keys = np.concatenate(parts)
    del parts
    return _csr_from_keys(m, k, keys, lambda n: rng.uniform(-1.0, 1.0, n).astype(np.float32), dtype)


def scrambled_band(m: int, seed: int, half_band: int = 13, dtype: str = F32) -> Csr:
    """A (2*half_band+1)-diagonal band whose rows and columns went through one random permutation: the
    structure a bandwidth-reducing reordering can restore (stand-in for a mesh matrix in arbitrary node order)."""
    rng = np.random.default_rng(seed)
    p = rng.permutation(m).astype(np.int64)
    i = np.arange(m, dtype=np.int64)
    parts = []
    for d in range(-half_band, half_band + 1):
        j = i + d
        ok = (j >= 0) & (j < m)
        parts.append(p[i[ok]] * m + p[j[ok]])
    keys = np.unique(np.concatenate(parts))
    return _csr_from_keys(m, m, keys, lambda n: rng.uniform(-1.0, 1.0, n).astype(np.float32), dtype)


# --------------------------------------------------------------------------
# named workloads (the five benchmark configurations and their variants).  `scale` < 1 shrinks them for tests.
# --------------------------------------------------------------------------
def workload_width(name: str) -> int:
    """Dense width N of a named workload without building its matrix ("_n<width>" overrides the default)."""
    mm = re.search(r"_n(\d+)(?:_|$)", name)
    if mm:
        return int(mm.group(1))
    raise KeyError(name)


def workload(name: str, scale: float = 1.0):
    """Return (csr, format, b_row, b_col, N, dtype, seedB) for a named workload.

    A suffix "_f32" or "_bf16" gives the same structure and the same random draws stored in the other
    precision (the dtype x format cross product; BCSR workloads default to bf16, WCSR ones to f32).
    """
    s = scale
    dt = None
    for suffix, d in (("_f32", F32), ("_bf16", BF16)):
        if name.endswith(suffix):
            name, dt = name[:-len(suffix)], d
    n_override = None   # "_n<width>": the same matrix against a dense operand of another width
    mm = re.match(r"^(.*)_n(\d+)$", name)
    if mm:
        name, n_override = mm.group(1), int(mm.group(2))
    h_override = None   # "_h<height>": a WCSR workload with another window height (before "_n", "_f32" / "_bf16")
    mm = re.match(r"^(wcsr_.*)_h(16|32|64)$", name)
    if mm:
        name, h_override = mm.group(1), int(mm.group(2))
    if n_override is not None or h_override is not None:
        w = list(workload(name + ("_" + dt if dt else ""), scale))
        if n_override is not None:
            w[4] = n_override
        if h_override is not None:
            w[2] = h_override
        return tuple(w)
    mm = re.match(r"^bcsr_sweep_b(32|64|128)_s(\d+)$", name)
    if mm:                              # config 5: long prefill, geometric block-row lengths
        b, pct = int(mm.group(1)), int(mm.group(2))
        m = max(4 * b, int(8192 * s))
        a = block_sparse_geometric(m, m, b, b, pct / 100.0, seed=1030 + b + pct, dtype=dt or BF16)
        return a, "bcsr", b, b, max(256, int(65536 * s)), dt or BF16, 1008
    blk = 128   # "_b64" / "_b32": the config-2 shapes pruned in smaller square blocks (same sparsity, own mask)
    for suffix, b in (("_b64", 64), ("_b32", 32)):
        if name.endswith(suffix) and name.startswith("bcsr_") and name != "bcsr_small" + suffix:
            name, blk = name[:-len(suffix)], b
    mm = re.match(r"^bcsr_gate_proj_s(\d+)$", name)
    if mm:                              # the case study's other sparsity levels (Section IV-D, kernel-level table)
        pct = int(mm.group(1))
        a = block_sparse_bernoulli(18944, 3584, blk, blk, pct / 100.0, seed=1040 + pct, dtype=dt or BF16)
        return a, "bcsr", blk, blk, max(256, int(16384 * s)), dt or BF16, 1005
    mm = re.match(r"^bcsr_gate_proj_k(\d+)$", name)
    if mm:                              # the projection's rows and sparsity with another inner dimension K
        kk = int(mm.group(1))
        a = block_sparse_bernoulli(18944, kk, blk, blk, 0.90, seed=1060, dtype=dt or BF16)
        return a, "bcsr", blk, blk, max(256, int(16384 * s)), dt or BF16, 1005
    if name == "bcsr_small":            # config 1
        a = block_sparse_bernoulli(1024, 1024, 64, 64, 0.90, seed=1001, dtype=dt or BF16)
        return a, "bcsr", 64, 64, 256, dt or BF16, 1004
    if name == "bcsr_gate_proj":        # config 2 (gate/up projection)
        a = block_sparse_bernoulli(18944, 3584, blk, blk, 0.90, seed=1002, dtype=dt or BF16)
        return a, "bcsr", blk, blk, max(256, int(16384 * s)), dt or BF16, 1005
    if name == "bcsr_down_proj":        # config 2 (down projection)
        a = block_sparse_bernoulli(3584, 18944, blk, blk, 0.90, seed=1012, dtype=dt or BF16)
        return a, "bcsr", blk, blk, max(256, int(16384 * s)), dt or BF16, 1015
    if name == "wcsr_zipf":             # config 3
        m = max(1024, int((1 << 20) * s))
        a = zipf_graph(m, m, 16 * m, seed=1003, dtype=dt or F32)
        return a, "wcsr", 16, 8, 128, dt or F32, 1006
    if name == "wcsr_band_dense_rows":  # config 4
        m = max(4096, int(2_000_000 * s))
        a = banded_plus_dense_rows(m, seed=1004, dense_row_nnz=max(64, int(200000 * s)), dtype=dt or F32)
        return a, "wcsr", 16, 8, 64, dt or F32, 1007
    if name == "wcsr_scrambled_band":   # reordering study (Section IV-A): bench.py's suffix _rcm reorders it first
        m = max(4096, int((1 << 20) * s))
        a = scrambled_band(m, seed=1021, dtype=dt or F32)
        return a, "wcsr", 16, 8, 128, dt or F32, 1022
    raise KeyError(name)
