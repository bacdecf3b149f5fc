"""The stream argument of the boundary: launches on a caller's non-NULL hipStream_t, concurrent calls on one handle
from two streams (the header promises that this is safe for handles that use no scratch), and the one-stream
ordering that calls sharing a handle's scratch must keep.  Streams are created at the default priority only.
Everything is checked against the oracle at the usual tolerances (bf16: 1e-2 * S + 1e-5, fp32: 1e-5 * S).
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


def _poisoned(shape, dtype):
    if dtype == "bf16":
        return torch.full(shape, 0x7FC1, dtype=torch.int16, device="cuda")
    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")


def _host(t, dtype):
    out = t.cpu().numpy()
    return out.view(np.uint16) if dtype == "bf16" else out


def _check(a, B, C):
    ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, a.dtype, B)
    got = synth.to_f64(C, a.dtype)
    assert np.isfinite(got).all(), "unwritten or non-finite output"
    bound = 1e-2 * S + 1e-5 if a.dtype == "bf16" else 1e-5 * S
    assert (np.abs(got - ref) <= bound).all()


def _side_stream():
    s = torch.cuda.Stream()        # default priority
    assert s.cuda_stream != 0      # a real hipStream_t, not the NULL stream
    return s


@pytest.mark.parametrize("fmt,dtype,b_row,b_col", [
    ("bcsr", "bf16", 128, 128), ("bcsr", "bf16", 64, 64), ("bcsr", "f32", 64, 64),
    ("wcsr", "f32", 16, 8), ("wcsr", "bf16", 32, 8),
])
def test_spmm_on_a_callers_stream(fmt, dtype, b_row, b_col):
    if fmt == "bcsr":
        a = synth.block_sparse_bernoulli(40 * 128, 5 * 128, b_row, b_col, 0.6, seed=601, dtype=dtype)
        N = 8 * 512
    else:
        a = synth.zipf_graph(6000, 6000, 14 * 6000, seed=602, cap=2500, dtype=dtype)
        N = 128
    B = synth.dense_normal(a.k, N, dtype, seed=603)
    Bd, Cd = _dev(B), _poisoned((a.m, N), dtype)
    h = asp.asp_create_from_csr(fmt, dtype, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
    try:
        asp.asp_reserve(h, N)
        torch.cuda.synchronize()   # operands were filled on the default stream
        s = _side_stream()
        asp.asp_spmm(h, Bd.data_ptr(), Cd.data_ptr(), N, s.cuda_stream)
        s.synchronize()
    finally:
        asp.asp_destroy(h)
    _check(a, B, _host(Cd, dtype))


@pytest.mark.parametrize("b", [128, 64])
def test_spmm_xt_on_a_callers_stream(b):
    a = synth.block_sparse_bernoulli(40 * 128, 5 * 128, b, b, 0.6, seed=604)
    N = 8 * 512 - 8
    X = synth.dense_normal(N, a.k, "bf16", seed=605)
    Xd, Yd = _dev(X), _poisoned((N, a.m), "bf16")
    h = asp.asp_create_from_csr("bcsr", "bf16", b, b, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        torch.cuda.synchronize()
        s = _side_stream()
        asp.asp_spmm_xt(h, Xd.data_ptr(), Yd.data_ptr(), N, s.cuda_stream)
        s.synchronize()
    finally:
        asp.asp_destroy(h)
    _check(a, np.ascontiguousarray(X.T), np.ascontiguousarray(_host(Yd, "bf16").T))


@pytest.mark.parametrize("fmt,dtype,b_row,b_col", [
    ("bcsr", "bf16", 128, 128),   # resident workgroups, static schedule: no shared mutable state
    ("bcsr", "bf16", 32, 32),
    ("bcsr", "f32", 128, 128),
    ("wcsr", "f32", 16, 8),       # no scratch reserved: split windows add into their own C with atomics
])
def test_two_streams_share_one_handle_concurrently(fmt, dtype, b_row, b_col):
    if fmt == "bcsr":
        a = synth.block_sparse_bernoulli(64 * 128, 6 * 128, b_row, b_col, 0.7, seed=611, dtype=dtype)
        N = 4096
    else:
        a = synth.zipf_graph(30000, 30000, 14 * 30000, seed=612, cap=4000, dtype=dtype)
        N = 128
    Bs = [synth.dense_normal(a.k, N, dtype, seed=613 + i) for i in range(2)]
    Bd = [_dev(B) for B in Bs]
    Cd = [_poisoned((a.m, N), dtype) for _ in range(2)]
    h = asp.asp_create_from_csr(fmt, dtype, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
    try:
        torch.cuda.synchronize()
        streams = [_side_stream(), _side_stream()]
        for _ in range(6):         # several calls per stream, issued alternately: the two queues overlap on the GPU
            for i in range(2):
                asp.asp_spmm(h, Bd[i].data_ptr(), Cd[i].data_ptr(), N, streams[i].cuda_stream)
        for s in streams:
            s.synchronize()
    finally:
        asp.asp_destroy(h)
    for i in range(2):
        _check(a, Bs[i], _host(Cd[i], dtype))


@pytest.mark.parametrize("dtype,b_row", [("bf16", 16), ("f32", 64)])
def test_calls_that_share_a_handles_scratch_ordered_on_one_stream(dtype, b_row):
    # the partial tiles of split windows go through the handle's one scratch buffer: the documented use is one
    # stream, where the second call's tasks start after the first call's sum kernel has read the buffer
    a = synth.zipf_graph(20000, 20000, 14 * 20000, seed=621, cap=4000, dtype=dtype)
    N = 128
    Bs = [synth.dense_normal(a.k, N, dtype, seed=622 + i) for i in range(3)]
    Bd = [_dev(B) for B in Bs]
    Cd = [_poisoned((a.m, N), dtype) for _ in range(3)]
    h = asp.asp_create_from_csr("wcsr", dtype, b_row, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
    try:
        assert asp.asp_get_info(h).n_zero_rows_units > 0
        asp.asp_reserve(h, N)
        torch.cuda.synchronize()
        s = _side_stream()
        for i in range(3):
            asp.asp_spmm(h, Bd[i].data_ptr(), Cd[i].data_ptr(), N, s.cuda_stream)
        s.synchronize()
    finally:
        asp.asp_destroy(h)
    for i in range(3):
        _check(a, Bs[i], _host(Cd[i], dtype))
