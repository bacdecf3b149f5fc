"""The launch paths under HIP graph capture: asp_spmm, asp_spmm_xt and asp_spmm_static_scratch issue kernels only
(no allocation, no memset, no host synchronisation), so a caller may record them into a graph.  Each case captures
one call, replays the graph three times -- the dense operand rewritten and the output poisoned by ordinary eager work
between the replays -- and compares every replay with an eager call on the same operands (bit for bit: all captured
paths are deterministic) and one of them with the oracle (bf16: 1e-2 * S + 1e-5, fp32: 1e-5 * S).
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


def _poison(t, dtype):
    if dtype == "bf16":
        t.fill_(0x7FC1)
    else:
        t.fill_(float("nan"))


def _host(t, dtype):
    out = t.cpu().numpy()
    return out.view(np.uint16) if dtype == "bf16" else out


CASES = [
    # (format, dtype, b_row, b_col, entry)
    ("bcsr", "bf16", 128, 128, "spmm"),        # 128 x 512-tile kernel
    ("bcsr", "bf16", 64, 64, "spmm"),          # composite form
    ("bcsr", "bf16", 128, 128, "xt"),          # K-contiguous entry
    ("bcsr", "f32", 64, 64, "spmm"),
    ("wcsr", "f32", 16, 8, "spmm"),            # split windows through the handle's scratch (three kernels per call)
    ("wcsr", "bf16", 32, 8, "spmm"),
    ("wcsr", "f32", 16, 8, "static_scratch"),  # the entry point that allocates nothing
]


@pytest.mark.parametrize("fmt,dtype,b_row,b_col,entry", CASES)
def test_captured_call_replays_like_the_eager_one(fmt, dtype, b_row, b_col, entry):
    if fmt == "bcsr":
        a = synth.block_sparse_bernoulli(40 * 128, 5 * 128, b_row, b_col, 0.6, seed=801, dtype=dtype)
        N = 8 * 512
    else:
        a = synth.zipf_graph(6000, 6000, 14 * 6000, seed=802, cap=2500, dtype=dtype)
        N = 128
    xt = entry == "xt"
    shape_b, shape_c = ((N, a.k), (N, a.m)) if xt else ((a.k, N), (a.m, N))
    tdt = torch.int16 if dtype == "bf16" else torch.float32
    Bs = [synth.dense_normal(shape_b[0], shape_b[1], dtype, seed=810 + r) for r in range(3)]
    Bd = _dev(Bs[0])
    Cd = torch.empty(shape_c, dtype=tdt, device="cuda")
    h = asp.asp_create_from_csr(fmt, dtype, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64)
    try:
        if entry != "static_scratch":
            asp.asp_reserve(h, N)                 # set-up: allocates the scratch of split windows, outside the capture
        call = {"spmm": asp.asp_spmm, "xt": asp.asp_spmm_xt, "static_scratch": asp.asp_spmm_static_scratch}[entry]

        def run():
            call(h, Bd.data_ptr(), Cd.data_ptr(), N, torch.cuda.current_stream().cuda_stream)

        run()                                     # once eagerly before capturing, as callers do
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run()
        for r in (1, 2, 0):
            Bd.copy_(_dev(Bs[r]))                 # eager work between the replays
            _poison(Cd, dtype)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            from_graph = _host(Cd, dtype).copy()
            _poison(Cd, dtype)
            run()
            torch.cuda.synchronize()
            eager = _host(Cd, dtype)
            assert np.array_equal(from_graph.view(np.uint8), eager.view(np.uint8)), "replay %d differs from the eager call" % r
        # the last replay (operand 0) against the oracle
        B0 = np.ascontiguousarray(Bs[0].T) if xt else Bs[0]
        C0 = np.ascontiguousarray(from_graph.T) if xt else from_graph
        ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, a.dtype, B0)
        got = synth.to_f64(C0, dtype)
        assert np.isfinite(got).all(), "unwritten or non-finite output"
        assert (np.abs(got - ref) <= (1e-2 * S + 1e-5 if dtype == "bf16" else 1e-5 * S)).all()
    finally:
        torch.cuda.synchronize()
        asp.asp_destroy(h)
