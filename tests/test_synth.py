"""The seeded generators produce valid, reproducible CSR inputs of the stated shape."""
import numpy as np
import pytest

from paper_2604_17834_amd import synth


def check_csr(a: synth.Csr):
    assert a.row_ptr.dtype == np.int32 and a.col_idx.dtype == np.int32
    assert a.row_ptr[0] == 0 and len(a.row_ptr) == a.m + 1 and a.row_ptr[-1] == len(a.col_idx) == len(a.values)
    assert np.all(np.diff(a.row_ptr) >= 0)
    if a.nnz:
        assert a.col_idx.min() >= 0 and a.col_idx.max() < a.k
        inner = np.ones(a.nnz, dtype=bool)
        inner[a.row_ptr[1:-1][a.row_ptr[1:-1] < a.nnz]] = False   # first entry of every row is exempt
        inner[0] = False
        assert np.all(np.diff(a.col_idx.astype(np.int64))[inner[1:]] > 0)   # strictly ascending inside rows


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, -2.0, 0.1, 3.1415927, 1e-30, 65504.0], dtype=np.float32)
    b = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(b)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert synth.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert synth.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


@pytest.mark.parametrize("gen", [synth.block_sparse_bernoulli, synth.block_sparse_geometric])
def test_block_masks(gen):
    a = gen(300, 200, 64, 64, 0.6, seed=3)
    b = gen(300, 200, 64, 64, 0.6, seed=3)
    check_csr(a)
    assert np.array_equal(a.col_idx, b.col_idx) and np.array_equal(a.values, b.values)
    # every touched 64x64 block is completely filled (ragged edges included)
    lens = np.diff(a.row_ptr)
    for I in range(5):
        rows = range(I * 64, min(300, I * 64 + 64))
        assert len({lens[r] for r in rows}) == 1
    v = synth.bf16_bits_to_f32(a.values)
    assert abs(v.std() - 0.02) < 0.002 and not (a.values == 0).any()


def test_zipf_graph():
    a = synth.zipf_graph(4096, 4096, 16 * 4096, seed=1, cap=500)
    check_csr(a)
    lens = np.diff(a.row_ptr)
    assert lens.max() <= 500 and lens.min() >= 1
    assert 0.85 * 16 * 4096 <= a.nnz <= 1.15 * 16 * 4096
    assert a.values.dtype == np.float32 and np.abs(a.values).max() <= 1.0
    assert np.median(lens) < lens.mean()           # heavy tail


def test_band_plus_dense_rows():
    a = synth.banded_plus_dense_rows(5000, seed=2, n_dense_rows=3, dense_row_nnz=800)
    check_csr(a)
    lens = np.diff(a.row_ptr)
    assert np.sort(lens)[-3] > 700 and np.sort(lens)[-4] <= 27
    i = 2500
    if lens[i] == 27:
        assert np.array_equal(a.col_idx[a.row_ptr[i]:a.row_ptr[i + 1]], np.arange(i - 13, i + 14))


def test_named_workloads_small():
    a, fmt, br, bc, N, dt, _ = synth.workload("bcsr_small")
    check_csr(a)
    assert (a.m, a.k, fmt, br, bc, N, dt) == (1024, 1024, "bcsr", 64, 64, 256, "bf16")
    a, fmt, br, bc, N, dt, _ = synth.workload("wcsr_zipf", scale=1 / 256)
    check_csr(a)
    assert (fmt, br, bc, N, dt) == ("wcsr", 16, 8, 128, "f32")
