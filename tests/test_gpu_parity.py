"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by element.

Tolerances (stated by the benchmark spec, written here):
  bf16 inputs, fp32 accumulation, bf16 output:  |C - C_ref| <= 1e-2 * S + 1e-5
  fp32 inputs and output:                       |C - C_ref| <= 1e-5 * S
with S = (|A| x |B|)_ij from the oracle.  Format arrays must be bit-exact.
"""
import numpy as np
import pytest

import oracle
from paper_2604_17834_amd import binding as asp
from paper_2604_17834_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _dev_in(x: np.ndarray):
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda()
    return torch.from_numpy(x).cuda()


def gpu_spmm(a: synth.Csr, fmt, b_row, b_col, B: np.ndarray, task_cols=0, handle=None, misalign=False, reserve=True):
    """One asp_create_from_csr + asp_spmm; returns C as numpy (uint16 bits or float32)."""
    own = handle is None
    if own:
        handle = asp.asp_create_from_csr(fmt, a.dtype, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values,
                                         task_cols=task_cols)
    try:
        N = B.shape[1]
        tdt = torch.int16 if a.dtype == "bf16" else torch.float32
        if misalign:  # shift both operands off 16-byte alignment by one element
            Bfull = torch.empty(B.size + 1, dtype=tdt, device="cuda")
            Bd = Bfull[1:].view(B.shape)
            Bd.copy_(_dev_in(np.ascontiguousarray(B)))
            Cfull = torch.empty(a.m * N + 1, dtype=tdt, device="cuda")
            Cd = Cfull[1:].view(a.m, N)
        else:
            Bd = _dev_in(np.ascontiguousarray(B))
            Cd = torch.empty((a.m, N), dtype=tdt, device="cuda")
        # poison C: every element must be overwritten (bf16 0x7FC1 / fp32 NaN)
        if a.dtype == "bf16":
            Cd.fill_(0x7FC1)
        else:
            Cd.fill_(float("nan"))
        stream = torch.cuda.current_stream().cuda_stream
        if reserve:   # scratch for the partial tiles of split WCSR windows; nothing for other handles
            asp.asp_reserve(handle, N)
        asp.asp_spmm(handle, Bd.data_ptr(), Cd.data_ptr(), N, stream)
        torch.cuda.synchronize()
        out = Cd.cpu().numpy()
        return out.view(np.uint16) if a.dtype == "bf16" else out
    finally:
        if own:
            asp.asp_destroy(handle)


def check_against_oracle(a: synth.Csr, B: np.ndarray, C: np.ndarray, cols=None):
    Bs = B if cols is None else np.ascontiguousarray(B[:, cols])
    Cs = C if cols is None else C[:, cols]
    ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, a.dtype, Bs)
    got = synth.to_f64(Cs, a.dtype)
    assert np.isfinite(got).all(), "unwritten or non-finite output"
    err = np.abs(got - ref)
    bound = 1e-2 * S + 1e-5 if a.dtype == "bf16" else 1e-5 * S
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), "worst at %s: got %r ref %r bound %r" % (worst, got[worst], ref[worst], bound[worst])
    return float((err / np.maximum(bound, 1e-300)).max())


# ------------------------------------------------------------------ BCSR
@pytest.mark.parametrize("b", [32, 64, 128])
@pytest.mark.parametrize("m,k,N,sparsity", [
    (256, 256, 256, 0.5),     # several tiles
    (384, 512, 64, 0.7),
    (300, 200, 128, 0.6),     # ragged M and K (last block row / column partly outside)
    (512, 384, 320, 0.8),     # N = 5 x 64: narrow tile chosen by the width rule
    (256, 256, 200, 0.5),     # masked N tail, 16-byte path (200 % 8 == 0)
    (160, 288, 100, 0.5),     # N % 8 != 0: element-wise path
    (128, 128, 8, 0.0),
    (128, 256, 1, 0.3),
])
def test_bcsr_parity(b, m, k, N, sparsity):
    a = synth.block_sparse_bernoulli(m, k, b, b, sparsity, seed=100 + b + N)
    B = synth.dense_normal(k, N, "bf16", seed=7 + N)
    C = gpu_spmm(a, "bcsr", b, b, B)
    check_against_oracle(a, B, C)


@pytest.mark.parametrize("b", [32, 64, 128])
def test_bcsr_scattered_entries_and_empty_block_rows(b):
    # unstructured entries: blocks are mostly zero padding; 30 % of rows empty => empty block-rows exist
    a = synth.random_csr(520, 390, 0.002, seed=b, dtype="bf16", empty_row_frac=0.3, dist="normal")
    B = synth.dense_normal(a.k, 136, "bf16", seed=1)
    C = gpu_spmm(a, "bcsr", b, b, B)
    check_against_oracle(a, B, C)
    empty = np.diff(a.row_ptr) == 0
    assert not C[empty].any()          # exactly +0


def test_bcsr_nnz_zero():
    a = synth.random_csr(100, 100, 0.0, seed=1, dtype="bf16")
    B = synth.dense_normal(100, 64, "bf16", seed=2)
    assert not gpu_spmm(a, "bcsr", 64, 64, B).any()


@pytest.mark.parametrize("b", [32, 64, 128])
def test_bcsr_times_identity_is_A_bit_exact(b):
    # products with 1.0 and sums with 0.0 are exact: the result must be A's bits, whatever the layout
    a = synth.random_csr(300, 256, 0.05, seed=10 + b, dtype="bf16", dist="normal")
    C = gpu_spmm(a, "bcsr", b, b, synth.dense_identity(a.k, "bf16"))
    dense = np.zeros((a.m, a.k), np.uint16)
    for i in range(a.m):
        dense[i, a.col_idx[a.row_ptr[i]:a.row_ptr[i + 1]]] = a.values[a.row_ptr[i]:a.row_ptr[i + 1]]
    assert np.array_equal(C, dense)


def test_bcsr_column_slice_and_rerun_bitwise():
    a = synth.block_sparse_geometric(512, 512, 64, 64, 0.7, seed=3)
    B = synth.dense_normal(a.k, 512, "bf16", seed=4)
    h = asp.asp_create_from_csr("bcsr", "bf16", 64, 64, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        C1 = gpu_spmm(a, "bcsr", 64, 64, B, handle=h)
        C2 = gpu_spmm(a, "bcsr", 64, 64, B, handle=h)
        assert np.array_equal(C1, C2)
        Cs = gpu_spmm(a, "bcsr", 64, 64, np.ascontiguousarray(B[:, 128:384]), handle=h)
        assert np.array_equal(C1[:, 128:384], Cs)
    finally:
        asp.asp_destroy(h)


def test_bcsr_misaligned_pointers_take_elementwise_path():
    a = synth.block_sparse_bernoulli(256, 256, 64, 64, 0.5, seed=5)
    B = synth.dense_normal(a.k, 64, "bf16", seed=6)
    C = gpu_spmm(a, "bcsr", 64, 64, B, misalign=True)
    check_against_oracle(a, B, C)


def test_bcsr_config1_full():
    a, fmt, br, bc, N, dt, seedB = synth.workload("bcsr_small")
    B = synth.dense_normal(a.k, N, dt, seedB)
    C = gpu_spmm(a, fmt, br, bc, B)
    check_against_oracle(a, B, C)


def _sample_columns(N, tile, rng):
    cols = list(range(0, 32)) + list(range(N - 32, N))
    for _ in range(2):
        s = int(rng.integers(1, N // tile - 1)) * tile + int(rng.integers(0, tile - 32))
        cols += list(range(s, s + 32))
    return np.array(sorted(set(cols)))


@pytest.mark.parametrize("name", ["bcsr_gate_proj", "bcsr_down_proj"])
def test_bcsr_config2_full_size_sampled_columns(name):
    # full benchmark shape on the GPU; every row checked on 128 sampled columns (a column of C
    # depends on the same column of B only, so the slice is an exact sub-problem for the oracle)
    a, fmt, br, bc, N, dt, seedB = synth.workload(name)
    B = synth.dense_normal(a.k, N, dt, seedB)
    C = gpu_spmm(a, fmt, br, bc, B)
    cols = _sample_columns(N, 256, np.random.default_rng(1))
    check_against_oracle(a, B, C, cols)
    # block-rows without blocks give exact zeros over the full width
    h = asp.asp_create_from_csr(fmt, dt, br, bc, a.m, a.k, a.row_ptr, a.col_idx, a.values,
                                flags=asp.ASP_FLAG_HOST_CONVERT_ONLY)
    brp = asp.asp_export(h, asp.ASP_ARR_ROW_PTR)
    asp.asp_destroy(h)
    for I in np.nonzero(np.diff(brp) == 0)[0]:
        assert not C[I * br:(I + 1) * br].any()


@pytest.mark.parametrize("b,sparsity", [(32, 0.9), (64, 0.75), (128, 0.95)])
def test_bcsr_geometric_rows_sampled(b, sparsity):
    # config-5 style: per-block-row length variance; reduced width so the oracle finishes in seconds
    a = synth.block_sparse_geometric(2048, 2048, b, b, sparsity, seed=50 + b)
    B = synth.dense_normal(a.k, 1024, "bf16", seed=51)
    C = gpu_spmm(a, "bcsr", b, b, B)
    check_against_oracle(a, B, C, _sample_columns(1024, 256, np.random.default_rng(2)))



# ---- 128 x 128 blocks with 512-wide tiles (chosen when every compute unit gets a tile) -------------------
def _plan_bn(a, N):
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        return asp.asp_plan_spmm(h, N).bn
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("m,k,N,sparsity", [
    (40 * 128, 5 * 128, 8 * 512, 0.5),             # aligned everywhere
    (40 * 128 + 40, 5 * 128 + 24, 8 * 512 - 8, 0.5),  # ragged M, K (last block column crosses K) and N tail
    (72 * 128, 128, 7 * 512, 0.2),                 # one block per block-row: every tile is a single block
    (64 * 128 + 8, 9 * 128, 4096, 0.85),           # very sparse: several block-rows stay empty
])
def test_bcsr_wide_tiles_parity(m, k, N, sparsity):
    a = synth.block_sparse_bernoulli(m, k, 128, 128, sparsity, seed=31, dtype="bf16")
    assert _plan_bn(a, N) == 512
    B = synth.dense_normal(k, N, "bf16", seed=32)
    C = gpu_spmm(a, "bcsr", 128, 128, B)
    check_against_oracle(a, B, C)


def test_bcsr_wide_tiles_empty_block_rows_and_rerun_bitwise():
    rng = np.random.default_rng(5)
    m, k, N = 48 * 128, 6 * 128, 4096
    a = synth.block_sparse_bernoulli(m, k, 128, 128, 0.6, seed=33, dtype="bf16")
    # empty out every fifth block-row
    keep = np.ones(a.nnz, dtype=bool)
    rows = np.repeat(np.arange(a.m), np.diff(a.row_ptr))
    keep[(rows // 128) % 5 == 2] = False
    rp = np.zeros(a.m + 1, dtype=np.int64)
    np.add.at(rp, rows[keep] + 1, 1)
    a2 = synth.Csr(a.m, a.k, np.cumsum(rp).astype(np.int32), a.col_idx[keep], a.values[keep], a.dtype)
    assert _plan_bn(a2, N) == 512
    B = synth.dense_normal(k, N, "bf16", seed=34)
    C1 = gpu_spmm(a2, "bcsr", 128, 128, B)
    C2 = gpu_spmm(a2, "bcsr", 128, 128, B)
    assert np.array_equal(C1, C2)
    assert not C1[2 * 128:3 * 128].any()  # an empty block-row: exact zeros
    cols = np.sort(rng.choice(N, 256, replace=False))
    check_against_oracle(a2, B, C1, cols)


def test_bcsr_wide_tiles_times_identity_is_A_bit_exact():
    m, k = 288 * 128, 512
    a = synth.block_sparse_bernoulli(m, k, 128, 128, 0.3, seed=35, dtype="bf16")
    N = 512
    assert _plan_bn(a, N) == 512 and k == N
    I = synth.dense_identity(k, "bf16")
    C = gpu_spmm(a, "bcsr", 128, 128, I)
    dense = np.zeros((m, k), dtype=np.uint16)
    rows = np.repeat(np.arange(m), np.diff(a.row_ptr))
    dense[rows, a.col_idx] = a.values
    dense[dense == 0x8000] = 0  # a stored -0.0 times 1.0, added to the +0.0 the sum starts from, is +0.0
    assert np.array_equal(C, dense)


# ---- 64 x 64 and 32 x 32 blocks through the composite form (128-row super-rows, four gathered K slices per block) --
def _plan_bn_b(a, b, N):
    h = asp.asp_create_from_csr("bcsr", "bf16", b, b, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        return asp.asp_plan_spmm(h, N).bn
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("b", [64, 32])
@pytest.mark.parametrize("m,k,N,sparsity,geometric", [
    (2560, 1024, 8192, 0.5, True),          # aligned everywhere
    (2560 - 40, 1024, 8192 + 72, 0.5, True),  # last block-row ragged (its second piece lies past M), N tail
    (4096, 2048, 4096, 0.3, False),         # dense-ish Bernoulli mask: nearly every strip is full
    (4096, 512, 4096 - 8, 0.6, False),
])
def test_bcsr_small_blocks_composite_parity(b, m, k, N, sparsity, geometric):
    k = k + b + (24 if sparsity == 0.6 else 0)   # a multiple of the block size but not of 128; one case of neither
    gen = synth.block_sparse_geometric if geometric else synth.block_sparse_bernoulli
    a = gen(m, k, b, b, sparsity, seed=61 + b, dtype="bf16")
    assert _plan_bn_b(a, b, N) == 512        # the composite form is in use
    B = synth.dense_normal(k, N, "bf16", seed=62)
    C = gpu_spmm(a, "bcsr", b, b, B)
    cols = np.r_[0:64, N // 2 - 32:N // 2 + 32, N - 64:N]
    check_against_oracle(a, B, C, cols)


@pytest.mark.parametrize("b", [64, 32])
def test_bcsr_small_blocks_composite_empty_rows_rerun_and_identity(b):
    m, k = 6144, 4096
    a = synth.block_sparse_bernoulli(m, k, b, b, 0.5, seed=63 + b, dtype="bf16")
    # empty out block-rows: single ones inside a super-row and two whole super-rows (rows 512..767)
    keep = np.ones(a.nnz, dtype=bool)
    rows = np.repeat(np.arange(a.m), np.diff(a.row_ptr))
    keep[((rows // b) % 7 == 3) | ((rows >= 512) & (rows < 768))] = False
    rp = np.zeros(a.m + 1, dtype=np.int64)
    np.add.at(rp, rows[keep] + 1, 1)
    a2 = synth.Csr(a.m, a.k, np.cumsum(rp).astype(np.int32), a.col_idx[keep], a.values[keep], a.dtype)
    N = k
    assert _plan_bn_b(a2, b, N) == 512
    I = synth.dense_identity(k, "bf16")
    C1 = gpu_spmm(a2, "bcsr", b, b, I)
    C2 = gpu_spmm(a2, "bcsr", b, b, I)
    assert np.array_equal(C1, C2)
    dense = np.zeros((m, k), dtype=np.uint16)
    dense[rows[keep], a2.col_idx] = a2.values
    dense[dense == 0x8000] = 0  # a stored -0.0 times 1.0, added to the +0.0 the sum starts from, is +0.0
    assert np.array_equal(C1, dense)
    assert not C1[512:768].any()


@pytest.mark.parametrize("entry", ["spmm", "xt"])
@pytest.mark.parametrize("b", [128, 64, 32])
def test_bcsr_mostly_empty_matrix_every_row_written(b, entry):
    # hundreds of block-rows without a stored block (more than the launch has workgroups): their rows of the
    # output are cleared in (span, part) items dealt over the workgroups, not span by span
    m, k, N = 400 * 128 + 24, 1024, 5 * 512 + 8
    a = synth.block_sparse_bernoulli(m, k, b, b, 0.97, seed=91 + b, dtype="bf16")
    lens = np.add.reduceat(np.diff(a.row_ptr), np.arange(0, m, b))
    assert (lens == 0).sum() * (b // 32 if b < 128 else 1) > 256
    empty = np.repeat(lens == 0, b)[:m]
    if entry == "spmm":
        assert _plan_bn_b(a, b, N) == 512
        B = synth.dense_normal(k, N, "bf16", seed=92)
        C = gpu_spmm(a, "bcsr", b, b, B)
    else:
        X = synth.dense_normal(N, k, "bf16", seed=92)
        B = np.ascontiguousarray(X.T)
        C = np.ascontiguousarray(gpu_spmm_xt(a, b, X).T)
    assert not C[empty].any()                                  # +0.0 in every column of every empty row
    assert not ((C & 0x7F80) == 0x7F80).any()                  # and no element left unwritten (the poison is a NaN)
    cols = np.r_[0:32, N // 2 - 16:N // 2 + 16, N - 32:N]
    check_against_oracle(a, B, C, cols)


@pytest.mark.parametrize("seed", range(12))
def test_bcsr_random_large_shapes_every_path(seed):
    # seeded random shapes large enough for the 128 x 512-tile kernel: every block size, ragged M / K / N, Bernoulli and
    # geometric masks from 30 % to 99.5 % block sparsity, both entries; whatever kernel the plan picks must match
    rng = np.random.default_rng(7000 + seed)
    b = int(rng.choice([128, 64, 32]))
    m = int(rng.integers(20, 300)) * 128 + int(rng.choice([0, 0, 8, 40, 64]))
    k = int(rng.integers(1, 16)) * 128 + int(rng.choice([0, 0, 32, 64]) if b < 128 else rng.choice([0, 0, 24]))
    N = int(rng.integers(1, 10)) * 512 + int(rng.choice([0, 0, 8, 72, 256]))
    sparsity = float(rng.choice([0.3, 0.7, 0.9, 0.97, 0.995]))
    gen = synth.block_sparse_geometric if rng.random() < 0.4 else synth.block_sparse_bernoulli
    xt = bool(rng.random() < 0.35)
    a = gen(m, k, b, b, sparsity, seed=7100 + seed, dtype="bf16")
    if xt:
        X = synth.dense_normal(N, k, "bf16", seed=7200 + seed)
        B = np.ascontiguousarray(X.T)
        C = np.ascontiguousarray(gpu_spmm_xt(a, b, X).T)
    else:
        B = synth.dense_normal(k, N, "bf16", seed=7200 + seed)
        C = gpu_spmm(a, "bcsr", b, b, B)
    assert not ((C & 0x7F80) == 0x7F80).any()                  # no element left unwritten (the poison is a NaN)
    lens = np.add.reduceat(np.diff(a.row_ptr), np.arange(0, a.m, b))
    assert not C[np.repeat(lens == 0, b)[:a.m]].any()          # rows of empty block-rows are +0.0 everywhere
    cols = np.unique(np.r_[0:16, rng.integers(0, N, 32), N - 16:N])
    check_against_oracle(a, B, C, cols)


@pytest.mark.parametrize("b", [64, 32])
def test_bcsr_small_blocks_composite_equals_small_block_kernel_within_rounding(b):
    # the same handle on a width where the composite form is not used (too few tiles) gives the same columns up
    # to the order of the fp32 sums: both must sit inside the oracle's bound, and mostly agree bit for bit
    a = synth.block_sparse_geometric(2560, 2048, b, b, 0.5, seed=65 + b, dtype="bf16")
    B = synth.dense_normal(a.k, 8192, "bf16", seed=66)
    h = asp.asp_create_from_csr("bcsr", "bf16", b, b, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        assert asp.asp_plan_spmm(h, 8192).bn == 512 and asp.asp_plan_spmm(h, 256).bn < 512   # the small-block kernel
        Cw = gpu_spmm(a, "bcsr", b, b, B, handle=h)
        Cn = gpu_spmm(a, "bcsr", b, b, np.ascontiguousarray(B[:, 1024:1280]), handle=h)
    finally:
        asp.asp_destroy(h)
    # parity: each kernel against the oracle
    check_against_oracle(a, np.ascontiguousarray(B[:, 1024:1280]), Cn)
    check_against_oracle(a, np.ascontiguousarray(B[:, 1024:1280]), Cw[:, 1024:1280])
    # not a parity claim, a diagnostic of the composite form: the two kernels add a row's products in different
    # orders, so they may differ in the last bit of some outputs, but an indexing mistake that still lands inside
    # the bound (two nearby columns swapped) would make them differ almost everywhere
    assert (Cw[:, 1024:1280] == Cn).mean() > 0.9


@pytest.mark.parametrize("b", [64, 32])
def test_bcsr_xt_small_blocks_composite_parity(b):
    m, k, N = 3072, 1024 + b, 8192 + 40
    a = synth.block_sparse_geometric(m, k, b, b, 0.5, seed=67 + b, dtype="bf16")
    # every fifth block-row empty: their outputs are cleared, in 64-byte pieces of the rows of Y
    keep = np.ones(a.nnz, dtype=bool)
    rows = np.repeat(np.arange(a.m), np.diff(a.row_ptr))
    keep[(rows // b) % 5 == 1] = False
    rp = np.zeros(a.m + 1, dtype=np.int64)
    np.add.at(rp, rows[keep] + 1, 1)
    a = synth.Csr(a.m, a.k, np.cumsum(rp).astype(np.int32), a.col_idx[keep], a.values[keep], a.dtype)
    assert _plan_bn_b(a, b, N) == 512
    X = synth.dense_normal(N, k, "bf16", seed=68)
    Y = gpu_spmm_xt(a, b, X)
    tok = np.r_[0:48, 4000:4048, N - 48:N]
    check_against_oracle(a, np.ascontiguousarray(X[tok].T), np.ascontiguousarray(Y[tok].T))
    # bit for bit the product of the transposed operands through asp_spmm (both take the composite path)
    C = gpu_spmm(a, "bcsr", b, b, np.ascontiguousarray(X.T))
    assert np.array_equal(Y, C.T)


# ---- K-contiguous entry: Y[N x m] = X[N x k] x A^T (Section IV-D's layout) -----------------------------------
def gpu_spmm_xt(a: synth.Csr, b, X: np.ndarray, misalign=False):
    h = asp.asp_create_from_csr("bcsr", a.dtype, b, b, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        N = X.shape[0]
        if misalign:
            Xf = torch.empty(X.size + 1, dtype=torch.int16, device="cuda")
            Xd = Xf[1:].view(X.shape)
            Xd.copy_(_dev_in(np.ascontiguousarray(X)))
            Yf = torch.empty(N * a.m + 1, dtype=torch.int16, device="cuda")
            Yd = Yf[1:].view(N, a.m)
        else:
            Xd = _dev_in(np.ascontiguousarray(X))
            Yd = torch.empty((N, a.m), dtype=torch.int16, device="cuda")
        Yd.fill_(0x7FC1)  # poison: every element must be overwritten
        asp.asp_spmm_xt(h, Xd.data_ptr(), Yd.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return Yd.cpu().numpy().view(np.uint16)
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("m,k,N,sparsity", [
    (40 * 128, 5 * 128, 8 * 512, 0.5),                # aligned everywhere: the MFMA path
    (40 * 128 + 40, 5 * 128 + 24, 8 * 512 - 13, 0.5),  # ragged M, K (chunks past K) and a token tail
    (72 * 128, 128, 7 * 512, 0.2),                    # single-block tiles
    (64 * 128 + 8, 9 * 128, 4096, 0.85),              # empty block-rows: their outputs are zero in every row of Y
])
def test_bcsr_xt_matrix_core_path_parity(m, k, N, sparsity):
    a = synth.block_sparse_bernoulli(m, k, 128, 128, sparsity, seed=41, dtype="bf16")
    X = synth.dense_normal(N, k, "bf16", seed=42)
    Y = gpu_spmm_xt(a, 128, X)
    # the definition: Y^T = A x X^T
    check_against_oracle(a, np.ascontiguousarray(X.T), np.ascontiguousarray(Y.T))


@pytest.mark.parametrize("b", [32, 64, 128])
@pytest.mark.parametrize("m,k,N,misalign", [(300, 200, 77, False), (256, 256, 64, True), (130, 96, 1, False)])
def test_bcsr_xt_generic_path_parity(b, m, k, N, misalign):
    a = synth.random_csr(m, k, 0.05, seed=43 + b, dtype="bf16", dist="normal", empty_row_frac=0.3)
    X = synth.dense_normal(N, k, "bf16", seed=44)
    Y = gpu_spmm_xt(a, b, X, misalign=misalign)
    check_against_oracle(a, np.ascontiguousarray(X.T), np.ascontiguousarray(Y.T))


@pytest.mark.parametrize("b,m,k,N", [
    (128, 256, 256, 64),        # 2 tiles: fewer than the 8 workgroups the launch never goes below
    (128, 128, 384, 8),         # one tile, 8 tokens
    (64, 640, 320, 200),        # smaller blocks on 128-row stacks, a token tail
    (128, 28 * 128, 1024, 1032),  # 28 block-rows x 3 token tiles, the last one 8 tokens wide
])
def test_bcsr_xt_matrix_core_path_with_fewer_tiles_than_compute_units(b, m, k, N):
    a = synth.block_sparse_bernoulli(m, k, b, b, 0.5, seed=48 + N, dtype="bf16")
    X = synth.dense_normal(N, k, "bf16", seed=49)
    Y = gpu_spmm_xt(a, b, X)
    check_against_oracle(a, np.ascontiguousarray(X.T), np.ascontiguousarray(Y.T))


@pytest.mark.parametrize("N", [1024, 4096])
def test_bcsr_xt_down_projection_at_short_sequences(N):
    # the case study's down projection (3584 x 18944, 28 block-rows) at sequence lengths where it has fewer
    # 128 x 512 tiles than the chip has compute units: still the matrix-core path
    a, fmt, br, bc, _, dt, seedB = synth.workload("bcsr_down_proj")
    X = synth.dense_normal(N, a.k, dt, seedB + N)
    Y = gpu_spmm_xt(a, br, X)
    tok = _sample_columns(N, 256, np.random.default_rng(6))
    check_against_oracle(a, np.ascontiguousarray(X[tok].T), np.ascontiguousarray(Y[tok].T))


def test_bcsr_xt_equals_transposed_spmm_bitwise():
    # both entries run the same multiply-add sequence per output on the matrix cores
    m, k, N = 48 * 128, 6 * 128, 4096
    a = synth.block_sparse_bernoulli(m, k, 128, 128, 0.6, seed=45, dtype="bf16")
    X = synth.dense_normal(N, k, "bf16", seed=46)
    Y = gpu_spmm_xt(a, 128, X)
    C = gpu_spmm(a, "bcsr", 128, 128, np.ascontiguousarray(X.T))
    assert np.array_equal(Y, C.T)


def test_bcsr_xt_rejects_wcsr_handles():
    a = synth.random_csr(64, 64, 0.1, seed=47, dtype="f32")
    h = asp.asp_create_from_csr("wcsr", "f32", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        x = torch.zeros((8, 64), dtype=torch.float32, device="cuda")
        y = torch.zeros((8, 64), dtype=torch.float32, device="cuda")
        assert asp.asp_spmm_xt(h, x.data_ptr(), y.data_ptr(), 8, None, check=False) == asp.ASP_ERR_UNSUPPORTED
    finally:
        asp.asp_destroy(h)

# ------------------------------------------------------------------ WCSR
@pytest.mark.parametrize("b_row", [16, 32, 64])
@pytest.mark.parametrize("m,k,N,density,task_cols", [
    (256, 300, 128, 0.05, 0),
    (200, 512, 64, 0.10, 16),      # splits: atomics + cleared rows
    (333, 257, 256, 0.03, 8),      # ragged last window, every window split
    (128, 128, 192, 0.10, 32),     # N = 3 x 64
    (100, 90, 100, 0.10, 16),      # masked N tail, 16-byte path
    (77, 140, 50, 0.15, 24),       # N % 4 != 0: element-wise path
    (64, 64, 4, 0.2, 0),
    (64, 64, 1, 0.2, 8),
])
def test_wcsr_parity(b_row, m, k, N, density, task_cols):
    a = synth.random_csr(m, k, density, seed=200 + m + N, dtype="f32", empty_row_frac=0.15)
    B = synth.dense_normal(k, N, "f32", seed=9 + N)
    C = gpu_spmm(a, "wcsr", b_row, 8, B, task_cols=task_cols)
    check_against_oracle(a, B, C)
    empty = np.diff(a.row_ptr) == 0
    assert not C[empty].any()


@pytest.mark.parametrize("b_row", [16, 32, 64])
def test_wcsr_times_identity_is_A_bit_exact(b_row):
    a = synth.random_csr(150, 128, 0.08, seed=20 + b_row, dtype="f32")
    C = gpu_spmm(a, "wcsr", b_row, 8, synth.dense_identity(a.k, "f32"), task_cols=16)
    dense = np.zeros((a.m, a.k), np.float32)
    for i in range(a.m):
        dense[i, a.col_idx[a.row_ptr[i]:a.row_ptr[i + 1]]] = a.values[a.row_ptr[i]:a.row_ptr[i + 1]]
    assert np.array_equal(C, dense)


def test_wcsr_empty_windows_and_nnz_zero():
    a = synth.random_csr(256, 200, 0.0, seed=1, dtype="f32")
    assert not gpu_spmm(a, "wcsr", 16, 8, synth.dense_normal(200, 64, "f32", 2)).any()
    a = synth.random_csr(256, 200, 0.05, seed=3, dtype="f32", empty_row_frac=0.9)  # many windows without columns
    B = synth.dense_normal(200, 128, "f32", 4)
    check_against_oracle(a, B, gpu_spmm(a, "wcsr", 16, 8, B))


def test_wcsr_unsplit_is_bitwise_reproducible_and_slice_consistent():
    a = synth.zipf_graph(4096, 4096, 16 * 4096, seed=8, cap=400)
    B = synth.dense_normal(a.k, 256, "f32", seed=9)
    h = asp.asp_create_from_csr("wcsr", "f32", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=1 << 20)
    try:
        assert asp.asp_get_info(h).n_zero_rows_units == np.count_nonzero(
            np.diff(asp.asp_export(h, asp.ASP_ARR_ROW_PTR)) == 0)
        C1 = gpu_spmm(a, "wcsr", 16, 8, B, handle=h)
        C2 = gpu_spmm(a, "wcsr", 16, 8, B, handle=h)
        assert np.array_equal(C1, C2)
        Cs = gpu_spmm(a, "wcsr", 16, 8, np.ascontiguousarray(B[:, 64:192]), handle=h)
        assert np.array_equal(C1[:, 64:192], Cs)
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("b_row,N", [(16, 128), (32, 100), (64, 50)])
def test_wcsr_f32_split_windows_without_scratch_use_atomics(b_row, N):
    # no asp_reserve: the tasks of a split window add into cleared rows of C with fp32 atomics
    a = synth.random_csr(200, 512, 0.10, seed=300 + b_row, dtype="f32", empty_row_frac=0.1)
    B = synth.dense_normal(a.k, N, "f32", seed=31)
    check_against_oracle(a, B, gpu_spmm(a, "wcsr", b_row, 8, B, task_cols=16, reserve=False))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_wcsr_split_windows_with_scratch_are_bitwise_reproducible(dtype):
    # partial tiles are added in task order: two runs give the same bits, and so does a wider reservation
    a = synth.zipf_graph(2048, 2048, 16 * 2048, seed=11, cap=900, dtype=dtype)
    B = synth.dense_normal(a.k, 128, dtype, seed=12)
    h = asp.asp_create_from_csr("wcsr", dtype, 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
    try:
        tasks = asp.asp_export(h, asp.ASP_ARR_TASKS)
        assert tasks[:, 3].any()
        C1 = gpu_spmm(a, "wcsr", 16, 8, B, handle=h)
        C2 = gpu_spmm(a, "wcsr", 16, 8, B, handle=h)
        assert np.array_equal(C1.view(np.uint8), C2.view(np.uint8))
        asp.asp_reserve(h, 512)
        C3 = gpu_spmm(a, "wcsr", 16, 8, B, handle=h)
        assert np.array_equal(C1.view(np.uint8), C3.view(np.uint8))
        check_against_oracle(a, B, C1)
    finally:
        asp.asp_destroy(h)


def test_wcsr_task_cols_does_not_change_result_beyond_tolerance():
    a = synth.zipf_graph(2048, 2048, 16 * 2048, seed=11, cap=900)
    B = synth.dense_normal(a.k, 128, "f32", seed=12)
    for tc in (8, 64, 512):
        check_against_oracle(a, B, gpu_spmm(a, "wcsr", 16, 8, B, task_cols=tc))


@pytest.mark.parametrize("b_row,task_cols", [(16, 64), (32, 8), (64, 512)])
def test_wcsr_device_arrays_and_gpu_task_partition_bit_exact(b_row, task_cols):
    # the task list of a device handle comes from the wavefront-scan kernels
    a = synth.zipf_graph(40000, 40000, 12 * 40000, seed=13, cap=5000)
    h = asp.asp_create_from_csr("wcsr", "f32", b_row, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=task_cols)
    try:
        wrp, wci, vals = oracle.to_wcsr(a.m, a.k, a.row_ptr, a.col_idx, a.values, "f32", b_row, 8)
        assert asp.asp_get_info(h).on_device == 1
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), wrp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), wci)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES).view(np.uint32), vals.view(np.uint32))
        tasks = oracle.wcsr_tasks(wrp, task_cols)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_TASKS), tasks)
        assert asp.asp_get_info(h).n_tasks == len(tasks)
    finally:
        asp.asp_destroy(h)


def test_bcsr_device_handle_exports_canonical_arrays():
    a = synth.block_sparse_bernoulli(512, 640, 128, 128, 0.6, seed=14)
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        brp, bci, blocks = oracle.to_bcsr(a.m, a.k, a.row_ptr, a.col_idx, a.values, "bf16", 128, 128)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), brp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), bci)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES), blocks)
    finally:
        asp.asp_destroy(h)


def test_wcsr_config3_full_size():
    # full irregular workload; the oracle does all 2^20 x 128 outputs
    a, fmt, br, bc, N, dt, seedB = synth.workload("wcsr_zipf")
    B = synth.dense_normal(a.k, N, dt, seedB)
    C = gpu_spmm(a, fmt, br, bc, B)
    check_against_oracle(a, B, C)


def test_wcsr_config4_reduced_band_plus_dense_rows():
    # band + long rows at 1/8 scale (long rows still span hundreds of tasks); N = 64 and 256
    a, fmt, br, bc, _, dt, seedB = synth.workload("wcsr_band_dense_rows", scale=0.125)
    for N in (64, 256):
        B = synth.dense_normal(a.k, N, dt, seedB + N)
        C = gpu_spmm(a, fmt, br, bc, B)
        cols = None if N == 64 else np.arange(96, 160)
        check_against_oracle(a, B, C, cols)


# ------------------------------------------------------------------ BCSR in fp32 (both formats at one precision)
@pytest.mark.parametrize("b", [32, 64, 128])
@pytest.mark.parametrize("m,k,N,sparsity", [
    (256, 256, 256, 0.5),     # several tiles, widest tile
    (384, 512, 128, 0.7),
    (300, 200, 384, 0.6),     # ragged M and K; N = 3 x 128
    (256, 384, 200, 0.5),     # masked N tail on the 16-byte path (200 % 4 == 0)
    (160, 288, 101, 0.5),     # N % 4 != 0: element-wise path
    (128, 256, 1, 0.3),
])
def test_bcsr_f32_parity(b, m, k, N, sparsity):
    a = synth.block_sparse_bernoulli(m, k, b, b, sparsity, seed=300 + b + N, dtype="f32", std=1.0)
    B = synth.dense_normal(k, N, "f32", seed=9 + N)
    C = gpu_spmm(a, "bcsr", b, b, B)
    check_against_oracle(a, B, C)


@pytest.mark.parametrize("b", [32, 64, 128])
def test_bcsr_f32_scattered_entries_identity_and_misalignment(b):
    a = synth.random_csr(520, 390, 0.004, seed=40 + b, dtype="f32", empty_row_frac=0.3, dist="normal")
    B = synth.dense_normal(a.k, 132, "f32", seed=2)
    C = gpu_spmm(a, "bcsr", b, b, B)
    check_against_oracle(a, B, C)
    assert not C[np.diff(a.row_ptr) == 0].any()      # rows without entries: exactly +0
    check_against_oracle(a, B, gpu_spmm(a, "bcsr", b, b, B, misalign=True))
    # products with 1.0 and sums with 0.0 are exact: A x I must be A's bits (a stored -0.0 adds up to +0.0)
    Ci = gpu_spmm(a, "bcsr", b, b, synth.dense_identity(a.k, "f32"))
    dense = np.zeros((a.m, a.k), np.float32)
    for i in range(a.m):
        dense[i, a.col_idx[a.row_ptr[i]:a.row_ptr[i + 1]]] = a.values[a.row_ptr[i]:a.row_ptr[i + 1]]
    assert np.array_equal(Ci.view(np.uint32), (dense + np.float32(0)).view(np.uint32))


def test_bcsr_f32_geometric_rows_sampled_and_rerun_bitwise():
    a = synth.block_sparse_geometric(2048, 2048, 128, 128, 0.9, seed=77, dtype="f32", std=1.0)
    B = synth.dense_normal(a.k, 1024, "f32", seed=78)
    h = asp.asp_create_from_csr("bcsr", "f32", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        C1 = gpu_spmm(a, "bcsr", 128, 128, B, handle=h)
        assert np.array_equal(C1, gpu_spmm(a, "bcsr", 128, 128, B, handle=h))
    finally:
        asp.asp_destroy(h)
    check_against_oracle(a, B, C1, _sample_columns(1024, 256, np.random.default_rng(3)))


# ------------------------------------------------------------------ WCSR in bf16 (both formats at one precision)
@pytest.mark.parametrize("b_row", [16, 32, 64])
@pytest.mark.parametrize("m,k,N,density,task_cols", [
    (256, 300, 128, 0.05, 0),      # one 128-column tile, no splits
    (200, 512, 64, 0.10, 16),      # N below the tile width; splits: fp32 scratch + final rounding
    (333, 257, 256, 0.03, 8),      # ragged last window, every window split, two tiles
    (128, 128, 200, 0.10, 32),     # masked N tail on the 16-byte path (200 % 8 == 0)
    (300, 700, 384, 0.20, 64),     # long windows: many stages per task, several tasks per window
    (77, 140, 50, 0.15, 24),       # N % 8 != 0: element-wise path
    (64, 64, 8, 0.2, 0),
    (64, 64, 1, 0.2, 8),
])
def test_wcsr_bf16_parity(b_row, m, k, N, density, task_cols):
    a = synth.random_csr(m, k, density, seed=400 + m + N, dtype="bf16", empty_row_frac=0.15)
    B = synth.dense_normal(k, N, "bf16", seed=19 + N)
    C = gpu_spmm(a, "wcsr", b_row, 8, B, task_cols=task_cols)
    check_against_oracle(a, B, C)
    assert not C[np.diff(a.row_ptr) == 0].any()


@pytest.mark.parametrize("b_row,task_cols", [(16, 16), (32, 1 << 20), (64, 40)])
def test_wcsr_bf16_times_identity_is_A_bit_exact(b_row, task_cols):
    # exact products and sums, and one rounding of an exactly representable value: split or not, A's bits come back
    a = synth.random_csr(150, 128, 0.08, seed=60 + b_row, dtype="bf16")
    C = gpu_spmm(a, "wcsr", b_row, 8, synth.dense_identity(a.k, "bf16"), task_cols=task_cols)
    dense = np.zeros((a.m, a.k), np.uint16)
    for i in range(a.m):
        dense[i, a.col_idx[a.row_ptr[i]:a.row_ptr[i + 1]]] = a.values[a.row_ptr[i]:a.row_ptr[i + 1]]
    dense[dense == 0x8000] = 0   # a stored -0.0 adds up to +0.0
    assert np.array_equal(C, dense)


def test_wcsr_bf16_pads_and_edges_never_read_B():
    # NaN rows of B that no stored column addresses, and a NaN-poisoned neighbourhood of the tile edge, must not leak:
    # pads and the columns past N load constants, not data
    a = synth.random_csr(96, 64, 0.12, seed=71, dtype="bf16")
    used = np.zeros(a.k, bool)
    used[a.col_idx] = True
    B = synth.dense_normal(a.k, 72, "bf16", seed=72)
    B[~used] = 0x7FC0
    C = gpu_spmm(a, "wcsr", 16, 8, B)
    B0 = B.copy()
    B0[~used] = 0
    check_against_oracle(a, B0, C)


def test_wcsr_bf16_unsplit_bitwise_reproducible_slices_and_misalignment():
    a = synth.zipf_graph(4096, 4096, 16 * 4096, seed=8, cap=400, dtype="bf16")
    B = synth.dense_normal(a.k, 256, "bf16", seed=9)
    h = asp.asp_create_from_csr("wcsr", "bf16", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=1 << 20)
    try:
        C1 = gpu_spmm(a, "wcsr", 16, 8, B, handle=h)
        assert np.array_equal(C1, gpu_spmm(a, "wcsr", 16, 8, B, handle=h))
        Cs = gpu_spmm(a, "wcsr", 16, 8, np.ascontiguousarray(B[:, 64:192]), handle=h)
        assert np.array_equal(C1[:, 64:192], Cs)
        # the element-wise path sums in a different order: same values within the tolerance
        check_against_oracle(a, B, gpu_spmm(a, "wcsr", 16, 8, B, handle=h, misalign=True))
        check_against_oracle(a, B, C1)
    finally:
        asp.asp_destroy(h)


def test_wcsr_bf16_scratch_must_be_reserved():
    a = synth.random_csr(64, 256, 0.5, seed=5, dtype="bf16")
    h = asp.asp_create_from_csr("wcsr", "bf16", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=32)
    try:
        B = torch.zeros((a.k, 128), dtype=torch.int16, device="cuda")
        C = torch.zeros((a.m, 128), dtype=torch.int16, device="cuda")
        assert asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), 128, None, check=False) == asp.ASP_ERR_BUFFER_TOO_SMALL
        assert "asp_reserve" in asp.asp_last_error()
        asp.asp_reserve(h, 64)
        assert asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), 128, None, check=False) == asp.ASP_ERR_BUFFER_TOO_SMALL
        assert asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), 64, None) == asp.ASP_OK     # smaller width fits
        asp.asp_reserve(h, 128)
        assert asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), 128, None) == asp.ASP_OK
        torch.cuda.synchronize()
    finally:
        asp.asp_destroy(h)


def test_wcsr_bf16_device_arrays_and_tasks_bit_exact():
    a = synth.zipf_graph(20000, 20000, 12 * 20000, seed=13, cap=5000, dtype="bf16")
    h = asp.asp_create_from_csr("wcsr", "bf16", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
    try:
        wrp, wci, vals = oracle.to_wcsr(a.m, a.k, a.row_ptr, a.col_idx, a.values, "bf16", 16, 8)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), wrp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), wci)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES).ravel(), vals.ravel())
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_TASKS), oracle.wcsr_tasks(wrp, 64))
    finally:
        asp.asp_destroy(h)


def test_wcsr_bf16_config3_full_size():
    a, fmt, br, bc, N, dt, seedB = synth.workload("wcsr_zipf_bf16")
    B = synth.dense_normal(a.k, N, dt, seedB)
    C = gpu_spmm(a, fmt, br, bc, B)
    check_against_oracle(a, B, C)


def test_wcsr_bf16_config4_reduced_band_plus_dense_rows():
    a, fmt, br, bc, _, dt, seedB = synth.workload("wcsr_band_dense_rows_bf16", scale=0.125)
    for N in (64, 256):
        B = synth.dense_normal(a.k, N, dt, seedB + N)
        C = gpu_spmm(a, fmt, br, bc, B)
        check_against_oracle(a, B, C, None if N == 64 else np.arange(96, 160))


# ------------------------------------------------------------------ reordering in front of the product (Section IV-A)
@pytest.mark.parametrize("fmt,b_row,b_col,dtype", [("wcsr", 16, 8, "f32"), ("bcsr", 32, 32, "bf16")])
def test_rcm_reordered_matrix_gives_the_permuted_product(fmt, b_row, b_col, dtype):
    a = synth.scrambled_band(3000, seed=5, half_band=9, dtype=dtype)
    perm = asp.asp_rcm(a.m, a.row_ptr, a.col_idx)
    rp, ci, va = asp.asp_permute_csr(a.m, a.k, a.row_ptr, a.col_idx, a.values, dtype, perm, perm)
    ar = synth.Csr(a.m, a.k, rp, ci, va, dtype)
    B = synth.dense_normal(a.k, 64, dtype, seed=6)
    Bp = np.ascontiguousarray(B[perm])
    Cr = gpu_spmm(ar, fmt, b_row, b_col, Bp)
    check_against_oracle(ar, Bp, Cr)                 # the reordered product against the oracle on the reordered matrix
    inv = np.empty_like(perm)
    inv[perm] = np.arange(a.m, dtype=perm.dtype)
    check_against_oracle(a, B, Cr[inv])              # ... and, rows put back, against the oracle on the original
    # the reordering did its job: far fewer stored units for the same entries
    h0 = asp.asp_create_from_csr(fmt, dtype, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=asp.ASP_FLAG_HOST_CONVERT_ONLY)
    h1 = asp.asp_create_from_csr(fmt, dtype, b_row, b_col, a.m, a.k, rp, ci, va, flags=asp.ASP_FLAG_HOST_CONVERT_ONLY)
    try:
        assert asp.asp_get_info(h1).n_units * 4 < asp.asp_get_info(h0).n_units
    finally:
        asp.asp_destroy(h0)
        asp.asp_destroy(h1)


def test_sparse_linear_layers_chain_without_transposes():
    # gate -> down of a small feed-forward block through the nn.Linear-shaped wrapper: every stage against the
    # oracle on the bf16 activations the previous stage produced
    from paper_2604_17834_amd.linear import SparseLinear
    N, hid, ffn = 512, 256, 1024
    wg = synth.block_sparse_bernoulli(ffn, hid, 128, 128, 0.5, seed=81, std=0.05)
    wd = synth.block_sparse_bernoulli(hid, ffn, 128, 128, 0.5, seed=82, std=0.05)
    gate = SparseLinear(ffn, hid, wg.row_ptr, wg.col_idx, wg.values)
    down = SparseLinear(hid, ffn, wd.row_ptr, wd.col_idx, wd.values)
    try:
        X = synth.dense_normal(N, hid, "bf16", seed=83)
        Xd = _dev_in(X)
        G = torch.full((N, ffn), 0x7FC1, dtype=torch.int16, device="cuda")
        Y = torch.full((N, hid), 0x7FC1, dtype=torch.int16, device="cuda")
        down(gate(Xd, G), Y)
        torch.cuda.synchronize()
        Gh, Yh = G.cpu().numpy().view(np.uint16), Y.cpu().numpy().view(np.uint16)
        check_against_oracle(wg, np.ascontiguousarray(X.T), np.ascontiguousarray(Gh.T))
        check_against_oracle(wd, np.ascontiguousarray(Gh.T), np.ascontiguousarray(Yh.T))
        with pytest.raises(ValueError):
            gate(Xd, Y)
    finally:
        gate.close()
        down.close()


def test_measurement_probes_run_and_count_their_work():
    # the benchmark's probe kernels live in a library of their own (not in the product's ABI)
    from paper_2604_17834_amd import measure
    out = torch.zeros(16, dtype=torch.float32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    stream = torch.cuda.current_stream().cuda_stream
    assert measure.asp_probe_mfma("bf16", 10, out.data_ptr(), stream) == 2 * cus * 4 * 10 * 8 * 2.0 * 32 * 32 * 16
    assert measure.asp_probe_mfma("f32", 10, out.data_ptr(), stream) == 2 * cus * 4 * 10 * 8 * 2.0 * 32 * 32 * 2
    x = torch.ones(1 << 20, dtype=torch.float32, device="cuda")
    measure.asp_probe_read(x.data_ptr(), x.numel() * 4, out.data_ptr(), stream)
    torch.cuda.synchronize()
    assert not out.any()                       # the probes never write their output in practice
    L = measure.lib()
    assert L.asp_probe_read(x.data_ptr() + 4, 64, out.data_ptr(), None) == 1
    assert L.asp_probe_mfma(7, 10, out.data_ptr(), None, None) == 1


# ------------------------------------------------------------------ the widened rows at the full benchmark shapes
@pytest.mark.parametrize("name", ["bcsr_gate_proj_f32", "bcsr_gate_proj_b64", "bcsr_down_proj_b32"])
def test_bcsr_other_precision_and_block_sizes_full_size_sampled_columns(name):
    a, fmt, br, bc, N, dt, seedB = synth.workload(name)
    B = synth.dense_normal(a.k, N, dt, seedB)
    C = gpu_spmm(a, fmt, br, bc, B)
    check_against_oracle(a, B, C, _sample_columns(N, 256, np.random.default_rng(4)))


def test_bcsr_xt_config2_full_size_sampled_tokens():
    # the K-contiguous entry at the benchmark shape: every output feature of 128 sampled tokens (first and last tile,
    # two interior slices) -- a token's outputs depend on that token's row of X only
    a, fmt, br, bc, N, dt, seedB = synth.workload("bcsr_gate_proj")
    X = synth.dense_normal(N, a.k, dt, seedB)
    Y = gpu_spmm_xt(a, br, X)
    tok = _sample_columns(N, 512, np.random.default_rng(5))
    check_against_oracle(a, np.ascontiguousarray(X[tok].T), np.ascontiguousarray(Y[tok].T))


@pytest.mark.parametrize("seed", range(48))
def test_random_configurations_parity(seed):
    # seeded draw over format, precision, sizes, density, block / window size, task size, alignment and scratch
    rng = np.random.default_rng(7000 + seed)
    fmt = str(rng.choice(["bcsr", "wcsr"]))
    dt = str(rng.choice(["bf16", "f32"]))
    m, k = int(rng.integers(1, 700)), int(rng.integers(1, 700))
    N = int(rng.choice([1, 3, 8, 17, 32, 64, 72, 100, 128, 136, 200, 256, 264, 384, 520]))
    dens = float(rng.choice([0.0, 0.002, 0.01, 0.05, 0.2, 0.6]))
    if fmt == "bcsr":
        br = bc = int(rng.choice([32, 64, 128]))
        tc = 0
    else:
        br, bc, tc = int(rng.choice([16, 32, 64])), 8, int(rng.choice([0, 8, 16, 40, 512]))
    mis = bool(rng.random() < 0.15)
    reserve = bool(rng.random() < 0.7) or dt == "bf16"
    a = synth.random_csr(m, k, dens, seed=8000 + seed, dtype=dt, empty_row_frac=float(rng.choice([0, 0.3])), dist="normal")
    B = synth.dense_normal(k, N, dt, seed=9000 + seed)
    C = gpu_spmm(a, fmt, br, bc, B, task_cols=tc, misalign=mis, reserve=reserve)
    check_against_oracle(a, B, C)


@pytest.mark.parametrize("seed", range(16))
def test_random_small_block_configurations_on_wide_tiles(seed):
    # seeded draw over the shapes that put 64x64 / 32x32 blocks on the 128x512-tile kernel (composite form):
    # block masks from dense to very sparse, empty block-rows, ragged M, any K that is a multiple of the block
    # size, N with and without a tail tile; both entries
    rng = np.random.default_rng(7100 + seed)
    b = int(rng.choice([32, 64]))
    m = int(rng.integers(2300, 6000))
    k = b * int(rng.integers(1, 40)) + 8 * int(rng.integers(0, 4))   # mostly with a partly filled last block column
    N = 8 * int(rng.integers(4096 // 8, 9000 // 8))
    sparsity = float(rng.choice([0.0, 0.3, 0.6, 0.8, 0.9, 0.97]))
    gen = synth.block_sparse_geometric if rng.random() < 0.5 else synth.block_sparse_bernoulli
    a = gen(m, k, b, b, sparsity, seed=7200 + seed, dtype="bf16")
    if rng.random() < 0.5:   # empty block-rows, singly and in runs
        keep = np.ones(a.nnz, dtype=bool)
        rows = np.repeat(np.arange(a.m), np.diff(a.row_ptr))
        brow = rows // b
        keep[(brow % 6 == 2) | ((brow >= 9) & (brow < 15))] = False
        rp = np.zeros(a.m + 1, dtype=np.int64)
        np.add.at(rp, rows[keep] + 1, 1)
        a = synth.Csr(a.m, a.k, np.cumsum(rp).astype(np.int32), a.col_idx[keep], a.values[keep], a.dtype)
    cols = np.sort(rng.choice(N, 96, replace=False))
    if rng.random() < 0.5 or m % 8 != 0:
        B = synth.dense_normal(k, N, "bf16", seed=7300 + seed)
        C = gpu_spmm(a, "bcsr", b, b, B)
        check_against_oracle(a, B, C, cols)
    else:
        X = synth.dense_normal(N, k, "bf16", seed=7300 + seed)
        Y = gpu_spmm_xt(a, b, X)
        check_against_oracle(a, np.ascontiguousarray(X[cols].T), np.ascontiguousarray(Y[cols].T))


def test_create_reserve_destroy_returns_device_memory():
    a = synth.zipf_graph(20000, 20000, 12 * 20000, seed=90, cap=3000, dtype="bf16")
    b = synth.block_sparse_bernoulli(1024, 1024, 64, 64, 0.7, seed=91)
    free0 = None
    for it in range(21):
        if it == 1:   # the first round also pays the runtime's one-time allocations
            torch.cuda.synchronize()
            free0 = torch.cuda.mem_get_info()[0]
        h = asp.asp_create_from_csr("wcsr", "bf16", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
        asp.asp_reserve(h, 64)
        asp.asp_reserve(h, 256)     # grows: the smaller buffer is freed
        asp.asp_destroy(h)
        h = asp.asp_create_from_csr("bcsr", "bf16", 64, 64, b.m, b.k, b.row_ptr, b.col_idx, b.values)
        asp.asp_destroy(h)
    torch.cuda.synchronize()
    assert abs(torch.cuda.mem_get_info()[0] - free0) < (8 << 20)
