"""Host-side checks of the C-ABI library (no GPU): symbols, argument errors, and the library's own
format converters bit for bit against the oracle's (host-convert mode makes no HIP call)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2604_17834_amd import binding as asp
from paper_2604_17834_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = asp.ASP_FLAG_HOST_CONVERT_ONLY


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "asyncsparse.h")).read()
    declared = set(re.findall(r"\b(asp_[a-z_]+)\s*\(", header))
    assert declared == set(asp.EXPORTED_SYMBOLS)
    L = asp.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_measurement_library_exports_its_header_and_nothing_of_it_is_in_the_product_abi():
    from paper_2604_17834_amd import measure
    header = open(os.path.join(ROOT, "include", "asyncsparse_measure.h")).read()
    declared = set(re.findall(r"\b(asp_[a-z_]+)\s*\(", header))
    assert declared == set(measure.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(measure.lib(), name) is not None
        assert not hasattr(asp.lib(), name)


def test_status_strings():
    assert asp.asp_status_string(0) == "ASP_OK"
    assert asp.asp_status_string(2) == "ASP_ERR_INVALID_CSR"
    assert asp.asp_status_string(99) == "ASP_ERR_UNKNOWN"


def _create_status(fmt, dtype, br, bc, m, k, rp, ci, va, task_cols=0, flags=HOST):
    st, h = asp.asp_create_from_csr(fmt, dtype, br, bc, m, k, rp, ci, va, task_cols, flags, check=False)
    if h:
        asp.asp_destroy(h)
    return st


def test_argument_and_csr_errors():
    rp = np.array([0, 1, 2], np.int32)
    ci = np.array([0, 1], np.int32)
    bf = np.array([1, 2], np.uint16)
    f32 = np.array([1, 2], np.float32)
    ok = _create_status("bcsr", "bf16", 32, 32, 2, 2, rp, ci, bf)
    assert ok == asp.ASP_OK
    assert _create_status("bcsr", "bf16", 48, 48, 2, 2, rp, ci, bf) == asp.ASP_ERR_UNSUPPORTED
    assert _create_status("bcsr", "bf16", 64, 32, 2, 2, rp, ci, bf) == asp.ASP_ERR_UNSUPPORTED
    assert _create_status("bcsr", "f32", 64, 64, 2, 2, rp, ci, f32) == asp.ASP_OK
    assert _create_status("bcsr", 5, 64, 64, 2, 2, rp, ci, f32) == asp.ASP_ERR_INVALID_ARG     # unknown dtype
    assert _create_status("wcsr", "f32", 16, 4, 2, 2, rp, ci, f32) == asp.ASP_ERR_UNSUPPORTED
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp, ci, f32, task_cols=12) == asp.ASP_ERR_INVALID_ARG
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp, ci, f32, task_cols=(1 << 30) + 8) == asp.ASP_ERR_INVALID_ARG
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp, ci, f32, task_cols=1 << 30) == asp.ASP_OK
    assert _create_status(7, "f32", 16, 8, 2, 2, rp, ci, f32) == asp.ASP_ERR_INVALID_ARG
    assert _create_status("wcsr", "f32", 16, 8, 0, 2, rp, ci, f32) == asp.ASP_ERR_INVALID_ARG
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp, ci, f32, flags=HOST | 8) == asp.ASP_ERR_INVALID_ARG
    # broken CSR
    bad = asp.ASP_ERR_INVALID_CSR
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, np.array([1, 1, 2], np.int32), ci, f32) == bad
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, np.array([0, 2, 1], np.int32), ci, f32) == bad
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, np.array([0, 1, 1], np.int32), ci, f32) == bad   # row_ptr[m] != nnz
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp, np.array([0, 2], np.int32), f32) == bad       # col >= k
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp, np.array([-1, 0], np.int32), f32) == bad
    rp2 = np.array([0, 2, 2], np.int32)
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp2, np.array([1, 0], np.int32), f32) == bad      # unsorted
    assert _create_status("wcsr", "f32", 16, 8, 2, 2, rp2, np.array([1, 1], np.int32), f32) == bad      # duplicate
    assert "ascending" in asp.asp_last_error()
    # null handle paths
    assert asp.lib().asp_get_info(None, None) == asp.ASP_ERR_INVALID_ARG
    assert asp.lib().asp_spmm(None, None, None, 4, None) == asp.ASP_ERR_INVALID_ARG
    assert asp.lib().asp_destroy(None) == asp.ASP_OK


def test_host_handle_refuses_spmm_and_small_export_buffer():
    a = synth.random_csr(40, 40, 0.1, 3, "f32")
    h = asp.asp_create_from_csr("wcsr", "f32", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        assert asp.asp_get_info(h).on_device == 0
        assert asp.lib().asp_spmm(h, 16, 32, 8, None) == asp.ASP_ERR_UNSUPPORTED
        assert asp.lib().asp_spmm(h, 16, 32, 0, None) == asp.ASP_ERR_INVALID_ARG
        need = ctypes.c_size_t()
        buf = np.zeros(1, np.int32)
        st = asp.lib().asp_export(h, asp.ASP_ARR_COL_IDX, buf.ctypes.data_as(ctypes.c_void_p), 4, ctypes.byref(need))
        assert st == asp.ASP_ERR_BUFFER_TOO_SMALL and need.value == 4 * asp.asp_get_info(h).n_units
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("m,k,br,density", [(64, 64, 32, 0.05), (200, 130, 32, 0.02), (129, 257, 64, 0.01),
                                            (300, 300, 128, 0.005), (31, 33, 32, 0.3), (128, 128, 64, 0.0)])
def test_bcsr_converter_bit_exact_vs_oracle(m, k, br, density):
    a = synth.random_csr(m, k, density, 5, "bf16", empty_row_frac=0.2, dist="normal")
    h = asp.asp_create_from_csr("bcsr", "bf16", br, br, m, k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        brp, bci, blocks = oracle.to_bcsr(m, k, a.row_ptr, a.col_idx, a.values, "bf16", br, br)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), brp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), bci)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES), blocks)
        info = asp.asp_get_info(h)
        assert (info.n_brows, info.n_units, info.nnz) == (len(brp) - 1, len(bci), a.nnz)
        assert info.fill_ratio == oracle.fill_ratio(a.nnz, len(bci), br, br)
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("m,k,br,density", [(200, 130, 32, 0.02), (129, 257, 64, 0.01), (300, 300, 128, 0.005)])
def test_bcsr_f32_converter_bit_exact_vs_oracle(m, k, br, density):
    a = synth.random_csr(m, k, density, 6, "f32", empty_row_frac=0.2, dist="normal")
    h = asp.asp_create_from_csr("bcsr", "f32", br, br, m, k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        brp, bci, blocks = oracle.to_bcsr(m, k, a.row_ptr, a.col_idx, a.values, "f32", br, br)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), brp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), bci)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES).view(np.uint32).ravel(), blocks.view(np.uint32).ravel())
        assert asp.asp_get_info(h).fill_ratio == oracle.fill_ratio(a.nnz, len(bci), br, br)
        for N in (128, 256, 384, 1024, 200, 101, 1):   # fp32 kernel: 128- and 256-wide tiles, element-wise at 128
            p = asp.asp_plan_spmm(h, N)
            assert p.vectorized == (1 if N % 4 == 0 else 0)
            assert p.bn == (oracle.choose_bn(N, [128, 256]) if N % 4 == 0 else 128)
            assert p.n_tiles == -(-N // p.bn) and p.workgroups == (len(brp) - 1) * p.n_tiles
    finally:
        asp.asp_destroy(h)


def test_bcsr_converter_block_mask_workload():
    a = synth.block_sparse_geometric(512, 768, 64, 64, 0.8, seed=9)
    h = asp.asp_create_from_csr("bcsr", "bf16", 64, 64, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        brp, bci, blocks = oracle.to_bcsr(a.m, a.k, a.row_ptr, a.col_idx, a.values, "bf16", 64, 64)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), brp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), bci)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES), blocks)
        assert asp.asp_get_info(h).fill_ratio == 1.0
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("m,k,br,density,task_cols", [(64, 64, 16, 0.05, 0), (200, 130, 16, 0.1, 16),
                                                      (129, 257, 32, 0.05, 8), (300, 300, 64, 0.02, 64),
                                                      (15, 33, 16, 0.5, 8), (128, 128, 16, 0.0, 0)])
def test_wcsr_converter_and_tasks_bit_exact_vs_oracle(m, k, br, density, task_cols):
    a = synth.random_csr(m, k, density, 6, "f32", empty_row_frac=0.2)
    h = asp.asp_create_from_csr("wcsr", "f32", br, 8, m, k, a.row_ptr, a.col_idx, a.values, task_cols=task_cols,
                                flags=HOST)
    try:
        wrp, wci, vals = oracle.to_wcsr(m, k, a.row_ptr, a.col_idx, a.values, "f32", br, 8)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), wrp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), wci)
        got = asp.asp_export(h, asp.ASP_ARR_VALUES)
        assert np.array_equal(got.view(np.uint32), vals.view(np.uint32))
        tc = task_cols or 512
        tasks = oracle.wcsr_tasks(wrp, tc)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_TASKS), tasks)
        info = asp.asp_get_info(h)
        assert (info.n_tasks, info.task_cols, info.n_units) == (len(tasks), tc, len(wci))
        widths = np.diff(wrp)
        assert info.n_zero_rows_units == np.count_nonzero((widths == 0) | (widths > tc))
    finally:
        asp.asp_destroy(h)


@pytest.mark.parametrize("br,task_cols", [(16, 16), (32, 0), (64, 24)])
def test_wcsr_bf16_converter_tasks_and_plan(br, task_cols):
    a = synth.random_csr(200, 257, 0.08, 8, "bf16", empty_row_frac=0.2)
    h = asp.asp_create_from_csr("wcsr", "bf16", br, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=task_cols,
                                flags=HOST)
    try:
        wrp, wci, vals = oracle.to_wcsr(a.m, a.k, a.row_ptr, a.col_idx, a.values, "bf16", br, 8)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), wrp)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), wci)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES).ravel(), vals.ravel())
        tasks = oracle.wcsr_tasks(wrp, task_cols or 512)
        assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_TASKS), tasks)
        for N in (128, 256, 200, 64, 8, 100, 1):   # one wave per (task, 128 columns), 4 waves to a workgroup
            p = asp.asp_plan_spmm(h, N)
            if N % 8 == 0:
                assert (p.vectorized, p.bn, p.n_tiles) == (1, 128, -(-N // 128))
                assert p.workgroups == -(-len(tasks) * p.n_tiles // 4)
            else:                                   # element-wise path: a workgroup per (window, 64 columns)
                assert (p.vectorized, p.bn, p.n_tiles) == (0, 64, -(-N // 64))
                assert p.workgroups == (len(wrp) - 1) * p.n_tiles
        assert asp.asp_reserve(h, 128, check=False) == asp.ASP_ERR_UNSUPPORTED   # no device arrays
    finally:
        asp.asp_destroy(h)
    assert asp.asp_reserve(None, 128, check=False) == asp.ASP_ERR_INVALID_ARG


def test_wcsr_converter_irregular_workloads():
    for a in (synth.zipf_graph(2048, 2048, 16 * 2048, seed=3, cap=700),
              synth.banded_plus_dense_rows(4096, seed=4, n_dense_rows=4, dense_row_nnz=1500)):
        h = asp.asp_create_from_csr("wcsr", "f32", 16, 8, a.m, a.k, a.row_ptr, a.col_idx, a.values, task_cols=64,
                                    flags=HOST)
        try:
            wrp, wci, vals = oracle.to_wcsr(a.m, a.k, a.row_ptr, a.col_idx, a.values, "f32", 16, 8)
            assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), wrp)
            assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), wci)
            assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES).view(np.uint32), vals.view(np.uint32))
            assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_TASKS), oracle.wcsr_tasks(wrp, 64))
        finally:
            asp.asp_destroy(h)


COST = [135, 96, 74, 64]   # the library's published cost per column of 64 / 128 / 256 / 512-wide tiles, in 1/64


def test_plan_follows_tile_width_rule():
    a = synth.block_sparse_bernoulli(256, 256, 128, 128, 0.5, 1)
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        for N in (64, 128, 192, 256, 320, 1024, 1104, 16384, 16448, 100, 72, 8, 1):
            p = asp.asp_plan_spmm(h, N)
            if N % 8 == 0:
                assert p.vectorized == 1
                assert p.bn == oracle.choose_bn_filled(N, [64, 128, 256], COST[:3], 2, 256)   # 2 block-rows, 256 units
            else:
                assert p.vectorized == 0 and p.bn == 64
            assert p.n_tiles == -(-N // p.bn) and p.padded_n == oracle.padded_width(N, p.bn)
            assert p.workgroups == 2 * p.n_tiles
    finally:
        asp.asp_destroy(h)
    # 128x128 blocks with at least one 512-wide tile per compute unit (256 assumed without a device): 512 joins the candidates
    a = synth.block_sparse_bernoulli(2048, 256, 128, 128, 0.0, 2)
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        for N, cands in ((16384, [64, 128, 256, 512]), (8192, [64, 128, 256, 512]), (4096, [64, 128, 256]), (8192 + 64, [64, 128, 256, 512]), (16448, [64, 128, 256, 512]), (1104, [64, 128, 256])):
            p = asp.asp_plan_spmm(h, N)
            assert p.bn == oracle.choose_bn_filled(N, cands, COST[:len(cands)], 16, 256), (N, p.bn)
        # a launch that would leave compute units without a tile takes narrower tiles: 16 block-rows need 16 tiles
        # along N to fill 256 units
        assert [asp.asp_plan_spmm(h, N).bn for N in (4096, 2048, 1024, 512, 64)] == [256, 128, 64, 64, 64]
    finally:
        asp.asp_destroy(h)
    # block-rows without a stored block are no tiles: they do not count
    a = synth.block_sparse_bernoulli(64 * 128, 256, 128, 128, 0.0, 2)
    keep = (np.repeat(np.arange(a.m), np.diff(a.row_ptr)) // 128) % 4 == 0      # 16 of 64 block-rows keep their blocks
    rp = np.zeros(a.m + 1, dtype=np.int64)
    np.add.at(rp, np.repeat(np.arange(a.m), np.diff(a.row_ptr))[keep] + 1, 1)
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, np.cumsum(rp).astype(np.int32), a.col_idx[keep],
                                a.values[keep], flags=HOST)
    try:
        assert [asp.asp_plan_spmm(h, N).bn for N in (4096, 2048, 1024)] == [256, 128, 64]
    finally:
        asp.asp_destroy(h)


def test_tile_width_costs_are_the_measured_time_ratios_and_the_rule_meets_the_papers_where_it_must():
    # the cost table the library ships (per column of a 64 / 128 / 256 / 512-wide tile, in 1/64 of the 512-wide
    # tile's) must be the ratios of the kernel times of the committed tile-width study (Section IV-C's experiment on
    # the projection workload), so that a re-measurement cannot leave the rule behind
    text = open(os.path.join(ROOT, "profiles", "bcsr_gate_proj_ablation.txt")).read()
    def kernel_ms(label):
        m = re.search(r"^" + re.escape(label) + r"\s+([0-9.]+)\s+[0-9.]+\s+(\d+)\s*$", text, re.M)
        assert m, label
        return float(m.group(1)), int(m.group(2))
    t512, bn512 = kernel_ms("+ 128x128 wave tiles, one wave per SIMD, hand-ordered issue, 128x512 tiles (default)")
    t256, bn256 = kernel_ms("+ direct-to-LDS ring, resident workgroups (2 per CU), static XCD-aware schedule, 128x256 tiles")
    t128, bn128 = kernel_ms("  same, 128x128 tiles")
    t64, bn64 = kernel_ms("  same, 128x64 tiles")
    assert (bn64, bn128, bn256, bn512) == (64, 128, 256, 512)
    # (box to box and run to run the ratios move by one or two units: the shipped table has to stay within 3)
    assert all(abs(round(64 * t / t512) - c) <= 3 for t, c in zip((t64, t128, t256, t512), COST))
    header = open(os.path.join(ROOT, "include", "asyncsparse.h")).read()
    assert "costs %d / %d / %d / %d" % tuple(COST) in header
    # Section IV-C's rule ("the largest width that divides N") and the shipped one agree whenever the widest
    # candidate divides N; the library's plan is checked against the paper's rule there
    a = synth.block_sparse_bernoulli(2048, 256, 128, 128, 0.0, 2)
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        for N in (8192, 16384, 65536, 512 * 33):
            assert asp.asp_plan_spmm(h, N).bn == oracle.choose_bn(N, [64, 128, 256, 512]) == 512
        # too few 512-wide tiles for every compute unit: 256 is the widest (and 16 x 16 tiles of it fill the 256 units)
        assert asp.asp_plan_spmm(h, 4096).bn == oracle.choose_bn(4096, [64, 128, 256]) == 256
    finally:
        asp.asp_destroy(h)


def test_plan_uses_wide_tiles_for_small_blocks_and_ragged_k():
    # 512-wide tiles need 128-row tiles: 128x128 blocks with K % 128 == 0, or the composite form (smaller blocks
    # within the fill limit; 128x128 blocks with a partly filled last block column) -- and a tile per compute unit
    cases = [
        (128, 40 * 128, 5 * 128, 0.5, 512),        # plain
        (128, 40 * 128, 5 * 128 + 24, 0.5, 512),   # ragged K: composite form without grouping
        (64, 40 * 128, 5 * 128 + 24, 0.5, 512),
        (32, 40 * 128, 5 * 128, 0.5, 512),
        (32, 40 * 128, 16, 0.0, 256),              # K below one slice: no composite form
        (64, 10 * 128, 5 * 128, 0.5, 256),         # too few tiles for every compute unit
    ]
    for b, m, k, sparsity, want in cases:
        a = synth.block_sparse_bernoulli(m, k, b, b, sparsity, 11)
        h = asp.asp_create_from_csr("bcsr", "bf16", b, b, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
        try:
            assert asp.asp_plan_spmm(h, 4096).bn == want, (b, m, k)
        finally:
            asp.asp_destroy(h)


def test_dense_width_limit_is_the_headers_and_is_enforced():
    hdr = open(os.path.join(os.path.dirname(__file__), "..", "include", "asyncsparse.h")).read()
    mm = re.search(r"#define ASP_MAX_N \((\d+)ll \* (\d+)\)", hdr)
    assert mm and int(mm.group(1)) * int(mm.group(2)) == asp.ASP_MAX_N
    a = synth.block_sparse_bernoulli(256, 256, 64, 64, 0.5, 4)
    h = asp.asp_create_from_csr("bcsr", "bf16", 64, 64, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        assert asp.asp_plan_spmm(h, asp.ASP_MAX_N).n_tiles >= 1
        with pytest.raises(asp.AspError) as e:
            asp.asp_plan_spmm(h, asp.ASP_MAX_N + 1)
        assert e.value.status == asp.ASP_ERR_INVALID_ARG
    finally:
        asp.asp_destroy(h)


def test_wcsr_conversion_does_not_depend_on_row_grouping():
    # the window's columns come from sorting its entries: rows with shared, disjoint and interleaved columns,
    # empty rows, a ragged last window, all window heights -- bit-exact against the oracle's converter
    rng = np.random.default_rng(77)
    m, k = 203, 5000
    rows = []
    for i in range(m):
        kind = i % 5
        if kind == 0:
            c = np.array([], np.int64)
        elif kind == 1:
            c = np.arange(0, 4000, 7)                      # shared by every such row
        elif kind == 2:
            c = np.arange(i, k, 211)                       # disjoint between rows
        elif kind == 3:
            c = np.sort(rng.choice(k, 300, replace=False))
        else:
            c = np.array([k - 1 - (i % 3)])
        rows.append(c)
    row_ptr = np.zeros(m + 1, np.int32)
    row_ptr[1:] = np.cumsum([len(c) for c in rows])
    col_idx = np.concatenate(rows).astype(np.int32)
    values = rng.uniform(-1, 1, len(col_idx)).astype(np.float32)
    for b_row in (16, 32, 64):
        wrp, wci, vals = oracle.to_wcsr(m, k, row_ptr, col_idx, values, "f32", b_row, 8)
        h = asp.asp_create_from_csr("wcsr", "f32", b_row, 8, m, k, row_ptr, col_idx, values, flags=HOST)
        try:
            assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_ROW_PTR), wrp)
            assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_COL_IDX), wci)
            assert np.array_equal(asp.asp_export(h, asp.ASP_ARR_VALUES).view(np.uint32).ravel(), vals.view(np.uint32).ravel())
        finally:
            asp.asp_destroy(h)


def test_spmm_entries_refuse_host_only_handles_and_null_pointers():
    a = synth.block_sparse_bernoulli(256, 256, 128, 128, 0.5, 3)
    h = asp.asp_create_from_csr("bcsr", "bf16", 128, 128, a.m, a.k, a.row_ptr, a.col_idx, a.values, flags=HOST)
    try:
        for fn in (asp.asp_spmm, asp.asp_spmm_xt):
            assert fn(h, 16, 32, 64, None, check=False) == asp.ASP_ERR_UNSUPPORTED   # no device arrays
            assert fn(h, None, 32, 64, None, check=False) == asp.ASP_ERR_INVALID_ARG
            assert fn(h, 16, 32, 0, None, check=False) == asp.ASP_ERR_INVALID_ARG
    finally:
        asp.asp_destroy(h)


def test_every_benchmarking_switch_has_a_gpu_parity_case():
    # the library reads its environment in exactly one place; every variable named there must be exercised by
    # tests/test_gpu_variants.py (one child process per setting, against the oracle)
    import glob
    srcs = {f: open(f).read() for f in glob.glob(os.path.join(ROOT, "paper_2604_17834_amd", "csrc", "*"))}
    readers = [f for f, text in srcs.items() if "getenv" in text]
    assert [os.path.basename(f) for f in readers] == ["asp_api.cpp"]
    names = set(re.findall(r'"(ASP_(?:BCSR|WCSR)_[A-Z_]+)"', srcs[readers[0]]))
    assert len(names) == 10
    cases = open(os.path.join(ROOT, "tests", "test_gpu_variants.py")).read()
    for n in names:
        assert '"%s"' % n in cases, n
