"""asp_spmm_static_scratch (the entry point for callers that cannot allocate) against asp_spmm with reserved scratch.

Both put the fp32 partial tiles of split WCSR windows into scratch memory and add them in task order, so their
outputs must agree bit for bit; the first is additionally checked against the oracle at the usual tolerances
(bf16: 1e-2 * S + 1e-5, fp32: 1e-5 * S).  Two calls in a row share the static array, the second with a smaller
input, so stale partial tiles of the first call lie in the slots the second one uses.
"""
import numpy as np
import pytest

import oracle
from paper_2604_17834_amd import binding as asp
from paper_2604_17834_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _dev(x):
    return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()


def _run(entry, h, a, B):
    N = B.shape[1]
    Bd = _dev(np.ascontiguousarray(B))
    Cd = torch.empty((a.m, N), dtype=torch.int16 if a.dtype == "bf16" else torch.float32, device="cuda")
    Cd.fill_(0x7FC1 if a.dtype == "bf16" else float("nan"))  # every element must be overwritten
    entry(h, Bd.data_ptr(), Cd.data_ptr(), N, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    out = Cd.cpu().numpy()
    return out.view(np.uint16) if a.dtype == "bf16" else out


def _check_oracle(a, B, C):
    ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, a.dtype, B)
    got = synth.to_f64(C, a.dtype)
    assert np.isfinite(got).all(), "unwritten or non-finite output"
    bound = 1e-2 * S + 1e-5 if a.dtype == "bf16" else 1e-5 * S
    assert (np.abs(got - ref) <= bound).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("b_row", [16, 64])
def test_static_scratch_matches_reserved_scratch_on_two_calls_in_a_row(dtype, b_row):
    # (rows, columns, entries, longest row, N): long rows make windows of several tasks (task_cols = 64)
    shapes = [(6144, 8192, 16 * 6144, 3000, 128), (1536, 4096, 12 * 1536, 900, 64)]
    for i, (m, k, nnz, cap, N) in enumerate(shapes):
        a = synth.zipf_graph(m, k, nnz, seed=70 + i, cap=cap, dtype=dtype)
        B = synth.dense_normal(k, N, dtype, seed=80 + i)
        h = asp.asp_create_from_csr("wcsr", dtype, b_row, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
        try:
            info = asp.asp_get_info(h)
            assert info.n_zero_rows_units > 0 and info.n_tasks > info.n_brows // 2
            got = _run(asp.asp_spmm_static_scratch, h, a, B)
            asp.asp_reserve(h, N)
            want = _run(asp.asp_spmm, h, a, B)
        finally:
            asp.asp_destroy(h)
        assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), "call %d differs from asp_spmm" % i
        _check_oracle(a, B, got)


def test_static_scratch_rejects_what_does_not_fit():
    # 4 * b_row * N bytes per task of a split window: 64 rows x 2^20 columns = 256 MiB per task
    a = synth.zipf_graph(2048, 4096, 16 * 2048, seed=90, cap=900, dtype="f32")
    h = asp.asp_create_from_csr("wcsr", "f32", 64, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
    try:
        one = torch.zeros(16, dtype=torch.float32, device="cuda")
        st = asp.asp_spmm_static_scratch(h, one.data_ptr(), one.data_ptr(), 1 << 20, None, check=False)
        assert st == asp.ASP_ERR_BUFFER_TOO_SMALL
        assert "static scratch" in asp.asp_last_error()
    finally:
        asp.asp_destroy(h)


def test_static_scratch_passes_bcsr_through():
    a = synth.block_sparse_bernoulli(512, 384, 128, 128, 0.6, seed=91)
    B = synth.dense_normal(a.k, 256, "bf16", seed=92)
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        got = _run(asp.asp_spmm_static_scratch, h, a, B)
        want = _run(asp.asp_spmm, h, a, B)
    finally:
        asp.asp_destroy(h)
    assert np.array_equal(got, want)
    _check_oracle(a, B, got)
