"""GPU parity where element and byte offsets pass 2^31: every kernel family once.

The index arrays are 32-bit (every workload has fewer than 2^31 stored entries), but products with the dense
width, the block area or the window height are not: C and B of these cases hold more than 2^31 elements (or
bytes), and one case has more than 2^31 stored tile values.  The dense operand is drawn on the device by a
seeded torch generator (it is too large to build on the host in reasonable time); the oracle gets the sampled
columns of exactly those bits, and a column of C depends on the same column of B only.
"""
import numpy as np
import pytest

import oracle
from paper_2604_17834_amd import binding as asp
from paper_2604_17834_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

WIDE = 1 << 21


def _device_normal(rows, cols, dtype, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.randn((rows, cols), dtype=tdt, device="cuda", generator=g)


def _bits(t):
    """Device tensor -> numpy in the oracle's storage type (bf16 as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def _poisoned(rows, cols, dtype):
    if dtype == "bf16":
        return torch.full((rows, cols), 0x7FC1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    return torch.full((rows, cols), float("nan"), dtype=torch.float32, device="cuda")


def _check(a, Bs, Cs):
    ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, a.dtype, Bs)
    got = synth.to_f64(Cs, a.dtype)
    assert np.isfinite(got).all(), "unwritten or non-finite output"
    bound = 1e-2 * S + 1e-5 if a.dtype == "bf16" else 1e-5 * S
    err = np.abs(got - ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), "worst at %s: got %r ref %r bound %r" % (worst, got[worst], ref[worst], bound[worst])


def _wide_columns(N):
    rng = np.random.default_rng(5)
    cols = list(range(0, 16)) + list(range(N - 16, N))
    for _ in range(3):
        s = int(rng.integers(1, N // 512 - 1)) * 512 + int(rng.integers(0, 512 - 16))
        cols += list(range(s, s + 16))
    return np.array(sorted(set(cols)))


@pytest.mark.parametrize("fmt,dtype,b_row,b_col", [
    ("bcsr", "bf16", 128, 128),   # 128x512 tiles, one wave per SIMD
    ("bcsr", "bf16", 64, 64),     # direct-to-LDS ring kernel for all block sizes
    ("bcsr", "f32", 128, 128),
    ("wcsr", "f32", 16, 8),
    ("wcsr", "bf16", 32, 8),
])
def test_dense_width_two_million_columns(fmt, dtype, b_row, b_col):
    # C: 1152 x 2^21 = 2.4e9 elements; B: 640 rows of 2^21 elements, rows from 512 (bf16: 1024) on start
    # beyond 2^31 bytes
    m, k, N = 1152, 640, WIDE
    if fmt == "bcsr":
        a = synth.block_sparse_bernoulli(m, k, b_row, b_col, 0.5, seed=901, dtype=dtype)
    else:
        a = synth.random_csr(m, k, 0.05, seed=902, dtype=dtype)   # 32 columns per row; windows of a few hundred
    print("case", fmt, dtype, b_row, "m", m, "k", k, "N", N, flush=True)
    B = _device_normal(k, N, dtype, seed=903)
    C = _poisoned(m, N, dtype)
    h = asp.asp_create_from_csr(fmt, dtype, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values,
                                task_cols=128 if fmt == "wcsr" else 0)     # several tasks per window
    try:
        asp.asp_reserve(h, N)
        asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        asp.asp_destroy(h)
    cols = _wide_columns(N)
    ct = torch.from_numpy(cols).cuda()
    _check(a, _bits(B[:, ct]), _bits(C[:, ct]))
    # every element was written: no poison left anywhere in the 2.4e9 outputs
    if dtype == "bf16":
        assert not bool((C.view(torch.int16) == 0x7FC1).any())
    else:
        assert not bool(torch.isnan(C).any())


@pytest.mark.parametrize("b", [128, 64])
def test_xt_two_million_tokens(b):
    # Y: 2^21 tokens x 1152 outputs, X: 2^21 x 640; token rows from 1.7 million on start beyond 2^31 bytes
    # (64x64 blocks: the same kernel on the composite form)
    m, k, N = 1152, 640, WIDE
    a = synth.block_sparse_bernoulli(m, k, b, b, 0.5, seed=904)
    print("case xt b", b, "m", m, "k", k, "tokens", N, flush=True)
    X = _device_normal(N, k, "bf16", seed=905)
    Y = _poisoned(N, m, "bf16")
    h = asp.asp_create_from_csr("bcsr", "bf16", b, b, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        asp.asp_spmm_xt(h, X.data_ptr(), Y.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        asp.asp_destroy(h)
    tok = torch.from_numpy(_wide_columns(N)).cuda()
    _check(a, np.ascontiguousarray(_bits(X[tok]).T), np.ascontiguousarray(_bits(Y[tok]).T))
    assert not bool((Y.view(torch.int16) == 0x7FC1).any())


@pytest.mark.parametrize("dtype,b_row", [("f32", 16), ("bf16", 16)])
def test_wcsr_seventeen_million_rows(dtype, b_row):
    # C: (2^24 + 4099) x 128 > 2^31 elements; two stored entries per row on average, a few long rows that split
    m, N = (1 << 24) + 4099, 128
    rng = np.random.default_rng(906)
    lens = rng.poisson(2.0, m).astype(np.int64)
    lens[rng.integers(0, m, 8)] = 3000                     # windows that split into tasks
    lens[m - 1] = 3000                                     # the last row, in the ragged last window
    row_ptr = np.zeros(m + 1, np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    nnz = int(row_ptr[-1])
    k = 1 << 16
    # ascending distinct columns per row: a random start plus distinct strides inside the row
    pos = np.arange(nnz, dtype=np.int64) - np.repeat(row_ptr[:-1], lens)
    start = np.repeat(rng.integers(0, k - 3000 * 16, m), lens)
    col_idx = (start + pos * 16 + rng.integers(0, 16, nnz)).astype(np.int32)
    vals = rng.uniform(-1.0, 1.0, nnz).astype(np.float32)
    values = synth.f32_to_bf16_bits(vals) if dtype == "bf16" else vals
    a = synth.Csr(m, k, row_ptr.astype(np.int32), col_idx, values, dtype)
    print("case wcsr rows", m, dtype, "nnz", nnz, flush=True)
    B = _device_normal(k, N, dtype, seed=907)
    C = _poisoned(m, N, dtype)
    h = asp.asp_create_from_csr("wcsr", dtype, b_row, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        asp.asp_reserve(h, N)
        asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        asp.asp_destroy(h)
    cols = np.r_[0:8, 60:68, 120:128]
    ct = torch.from_numpy(cols).cuda()
    _check(a, _bits(B[:, ct]), _bits(C[:, ct]))
    if dtype == "bf16":
        assert not bool((C.view(torch.int16) == 0x7FC1).any())
    else:
        assert not bool(torch.isnan(C).any())


def test_wcsr_more_than_two_billion_tile_values():
    # window height 64: 35.7 million packed columns x 64 rows = 2.28e9 stored tile values (9.1 GB in fp32)
    m, k, N = 1 << 21, 1 << 20, 64
    rng = np.random.default_rng(908)
    per_row = 17
    # row r of a window takes columns base(window) + r + 64 j, j < 17: ascending in the row, disjoint between the
    # rows of the window, so every window has 64 x 17 = 1088 packed columns: 32768 x 1088 = 35.7e6
    r = np.arange(m, dtype=np.int64)
    base = ((r // 64) * 977) % (k - 64 * per_row) + r % 64
    col_idx = (base[:, None] + 64 * np.arange(per_row, dtype=np.int64)[None, :]).astype(np.int32).ravel()
    row_ptr = (np.arange(m + 1, dtype=np.int64) * per_row).astype(np.int32)
    values = rng.uniform(-1.0, 1.0, m * per_row).astype(np.float32)
    a = synth.Csr(m, k, row_ptr, col_idx, values, "f32")
    print("case wcsr tile values, rows", m, "nnz", m * per_row, flush=True)
    h = asp.asp_create_from_csr("wcsr", "f32", 64, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        info = asp.asp_get_info(h)
        assert info.n_units * 64 > (1 << 31), info.n_units
        B = _device_normal(k, N, "f32", seed=909)
        C = _poisoned(m, N, "f32")
        asp.asp_reserve(h, N)
        asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        asp.asp_destroy(h)
    cols = np.r_[0:8, 56:64]
    ct = torch.from_numpy(cols).cuda()
    _check(a, _bits(B[:, ct]), _bits(C[:, ct]))
    assert not bool(torch.isnan(C).any())
