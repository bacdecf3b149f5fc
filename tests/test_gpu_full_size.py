"""GPU parity at the full sizes of the irregular-matrix and long-prefill workloads, in the launch configuration
that bench.py times (default task size, default tile-width rule, 16-byte aligned operands).

  band + dense rows (stand-in for the sparse-matrix evaluation, Section IV-A): 2e6 x 2e6, 27 diagonals plus 64
      rows of 200 000 random columns, window height 16, N = 64 (every output) and N = 256 (sampled columns),
      fp32 and bf16;
  long prefill (Section IV-D, sequence lengths up to 64K tokens): 8192 x 8192 in 128 / 64 / 32 blocks with
      geometric block-row lengths, N = 65536, all rows on sampled columns.

The dense operand is drawn on the device by a seeded torch generator; the oracle gets the sampled columns of
exactly those bits (a column of C depends on the same column of B only).  Tolerances as everywhere:
bf16 |C - C_ref| <= 1e-2 * S + 1e-5, fp32 <= 1e-5 * S, S = (|A| x |B|)_ij from the oracle.
"""
import numpy as np
import pytest

import oracle
from paper_2604_17834_amd import binding as asp
from paper_2604_17834_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _device_normal(rows, cols, dtype, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.randn((rows, cols), dtype=tdt, device="cuda", generator=g)


def _bits(t):
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def _poisoned(rows, cols, dtype):
    if dtype == "bf16":
        return torch.full((rows, cols), 0x7FC1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    return torch.full((rows, cols), float("nan"), dtype=torch.float32, device="cuda")


def _no_poison_left(C):
    if C.dtype == torch.bfloat16:
        return not bool((C.view(torch.int16) == 0x7FC1).any())
    return not bool(torch.isnan(C).any())


def _check(a, Bs, Cs):
    ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, a.dtype, Bs)
    got = synth.to_f64(Cs, a.dtype)
    assert np.isfinite(got).all(), "unwritten or non-finite output"
    bound = 1e-2 * S + 1e-5 if a.dtype == "bf16" else 1e-5 * S
    err = np.abs(got - ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), "worst at %s: got %r ref %r bound %r" % (worst, got[worst], ref[worst], bound[worst])


def _column_slices(N, width, interior, seed):
    """First and last `width` columns plus `interior` seeded slices of the same width (sorted, distinct)."""
    rng = np.random.default_rng(seed)
    cols = list(range(width)) + list(range(N - width, N))
    for _ in range(interior):
        s = int(rng.integers(width, N - 2 * width))
        cols += list(range(s, s + width))
    return np.array(sorted(set(cols)))


# ------------------------------------------------------------------ band + 64 dense rows at full size
@pytest.fixture(scope="module", params=["f32", "bf16"])
def band_handle(request):
    dtype = request.param
    name = "wcsr_band_dense_rows" + ("_bf16" if dtype == "bf16" else "")
    a, fmt, br, bc, _, dt, seedB = synth.workload(name)
    assert (a.m, fmt, br, bc, dt) == (2_000_000, "wcsr", 16, 8, dtype)
    print("case band_dense_rows", dtype, "m", a.m, "nnz", a.nnz, flush=True)
    h = asp.asp_create_from_csr(fmt, dt, br, bc, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    yield a, h, seedB
    asp.asp_destroy(h)


@pytest.mark.parametrize("N", [64, 256])
def test_band_plus_dense_rows_full_size(band_handle, N):
    a, h, seedB = band_handle
    info = asp.asp_get_info(h)
    assert info.n_tasks > info.n_brows + 64 * 300      # the 64 long rows split into hundreds of tasks each
    print("case band_dense_rows", a.dtype, "N", N, "tasks", info.n_tasks, flush=True)
    B = _device_normal(a.k, N, a.dtype, seed=seedB + N)
    C = _poisoned(a.m, N, a.dtype)
    asp.asp_reserve(h, N)
    asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert _no_poison_left(C)
    if N == 64:
        _check(a, _bits(B), _bits(C))                  # every output
    else:
        ct = torch.from_numpy(_column_slices(N, 16, 2, seed=4)).cuda()
        _check(a, _bits(B[:, ct]), _bits(C[:, ct]))


# ------------------------------------------------------------------ long prefill: 8192 x 8192, N = 65536
PREFILL_N = 65536


@pytest.fixture(scope="module")
def prefill_operands():
    B = _device_normal(8192, PREFILL_N, "bf16", seed=1008)
    C = _poisoned(8192, PREFILL_N, "bf16")
    yield B, C


@pytest.mark.parametrize("b,pct,wide", [
    (128, 50, True), (128, 90, True), (128, 99, True),   # 128x512 tiles on the handle's own blocks
    (64, 50, True), (64, 99, None),                        # 128-row stacks of smaller blocks where the handle keeps them
    (32, 50, True), (32, 99, None),
])
def test_long_prefill_geometric_block_rows_full_size(prefill_operands, b, pct, wide):
    B, C = prefill_operands
    a, fmt, br, bc, N, dt, _ = synth.workload("bcsr_sweep_b%d_s%d" % (b, pct))
    assert (a.m, a.k, N, fmt, br, dt) == (8192, 8192, PREFILL_N, "bcsr", b, "bf16")
    C.view(torch.int16).fill_(0x7FC1)
    h = asp.asp_create_from_csr(fmt, dt, br, bc, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        plan = asp.asp_plan_spmm(h, N)
        print("case long_prefill b", b, "sparsity", pct, "nnz", a.nnz, "bn", plan.bn, flush=True)
        if wide:
            assert plan.bn == 512        # geometric block-row lengths on the 128 x 512-tile kernel
        asp.asp_spmm(h, B.data_ptr(), C.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        asp.asp_destroy(h)
    assert _no_poison_left(C)
    ct = torch.from_numpy(_column_slices(N, 32, 2, seed=b + pct)).cuda()
    _check(a, _bits(B[:, ct]), _bits(C[:, ct]))
