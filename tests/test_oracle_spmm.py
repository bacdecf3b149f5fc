"""Pins for the oracle's product C = A x B (Section II-C): things the mathematics fixes.

None of these re-type the oracle's own loop: brute force goes through a
densified A and a triple loop, the library cross-check goes through scipy, the
rest are closed forms and invariants.
"""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2604_17834_amd import synth


def densify(a: synth.Csr) -> np.ndarray:
    d = np.zeros((a.m, a.k), dtype=np.float64)
    v = synth.to_f64(a.values, a.dtype)
    for i in range(a.m):
        for p in range(a.row_ptr[i], a.row_ptr[i + 1]):
            d[i, a.col_idx[p]] = v[p]
    return d


def brute_gemm(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    m, k = A.shape
    n = B.shape[1]
    C = np.zeros((m, n), dtype=np.float64)
    for i in range(m):
        for j in range(n):
            acc = 0.0
            for t in range(k):
                acc += A[i, t] * B[t, j]
            C[i, j] = acc
    return C


def run(a: synth.Csr, B):
    return oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, a.dtype, B)


def test_golden_worked_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "formats_4x6_example.json")))
    C, S = oracle.spmm(g["m"], g["k"], np.array(g["row_ptr"]), np.array(g["col_idx"]),
                       np.array(g["values"], dtype=np.float32), "f32", np.array(g["B"], dtype=np.float32))
    assert np.array_equal(C, np.array(g["C"], dtype=np.float64))
    assert np.array_equal(S, C)  # all entries positive => |A||B| = AB


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m,k,n,density,seed", [
    (1, 1, 1, 1.0, 1), (7, 5, 3, 0.5, 2), (33, 40, 17, 0.2, 3), (64, 64, 9, 0.05, 4), (20, 31, 5, 0.0, 5)])
def test_vs_dense_brute_force(dtype, m, k, n, density, seed):
    a = synth.random_csr(m, k, density, seed, dtype, empty_row_frac=0.2 if m > 4 else 0.0)
    B = synth.dense_normal(k, n, dtype, seed + 100)
    C, S = run(a, B)
    Ad, Bd = densify(a), synth.to_f64(B, dtype)
    ref = brute_gemm(Ad, Bd)
    refS = brute_gemm(np.abs(Ad), np.abs(Bd))
    assert np.allclose(C, ref, rtol=0, atol=1e-13 * max(1.0, refS.max()))
    assert np.allclose(S, refS, rtol=1e-13, atol=0)
    # rows without entries are exactly zero
    empty = np.diff(a.row_ptr) == 0
    assert not C[empty].any() and not S[empty].any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_times_identity_is_A_exactly(dtype):
    a = synth.random_csr(50, 37, 0.15, 11, dtype)
    C, _ = run(a, synth.dense_identity(a.k, dtype))
    assert np.array_equal(C, densify(a))


def test_linearity_in_B():
    a = synth.random_csr(60, 45, 0.1, 21, "f32")
    B1 = synth.dense_normal(a.k, 8, "f32", 22)
    B2 = synth.dense_normal(a.k, 8, "f32", 23)
    # alpha, beta powers of two and B1+B2 formed in fp32 exactly representable? not in general:
    # build the combination in fp64 and feed fp32 inputs that are exact: use alpha=2, beta=-0.5 on
    # operands whose sum is exact by construction (B2 = multiple of a coarse grid).
    B1 = np.round(B1 * 64) / 64
    B2 = np.round(B2 * 64) / 64
    comb = (2.0 * B1 - 0.5 * B2).astype(np.float32)
    assert np.array_equal(comb.astype(np.float64), 2.0 * B1.astype(np.float64) - 0.5 * B2.astype(np.float64))
    C1, S1 = run(a, B1.astype(np.float32))
    C2, S2 = run(a, B2.astype(np.float32))
    Cc, _ = run(a, comb)
    assert np.allclose(Cc, 2.0 * C1 - 0.5 * C2, rtol=0, atol=1e-13 * (2 * S1 + 0.5 * S2).max())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_vs_scipy_float64(dtype):
    a = synth.random_csr(300, 257, 0.03, 31, dtype, empty_row_frac=0.1)
    B = synth.dense_normal(a.k, 24, dtype, 32)
    C, S = run(a, B)
    M = sp.csr_matrix((synth.to_f64(a.values, dtype), a.col_idx, a.row_ptr), shape=(a.m, a.k))
    ref = M @ synth.to_f64(B, dtype)
    assert np.allclose(C, ref, rtol=0, atol=1e-12 * S.max())
    refS = abs(M) @ np.abs(synth.to_f64(B, dtype))
    assert np.allclose(S, refS, rtol=1e-12)


def test_column_slice_is_exact_subproblem():
    # column j of C depends on column j of B only: a slice of B gives the same columns bit for bit
    a = synth.random_csr(40, 30, 0.2, 41, "f32")
    B = synth.dense_normal(a.k, 16, "f32", 42)
    C, _ = run(a, B)
    Cs, _ = run(a, np.ascontiguousarray(B[:, 5:11]))
    assert np.array_equal(C[:, 5:11], Cs)


def test_bf16_widening_is_exact():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1 (bf16), 0x0001 = smallest subnormal
    bits = np.array([0x3F80, 0xC000, 0x3DCD, 0x0001], dtype=np.uint16)
    C, _ = oracle.spmm(1, 4, np.array([0, 4]), np.arange(4), bits, "bf16",
                       synth.dense_identity(4, "bf16"))
    expect = np.array([1.0, -2.0, 0.10009765625, 2.0 ** -133])
    assert np.array_equal(C[0], expect)


def test_sign_and_order_sensitivity():
    # a transposed operand or a wrong sign would change this asymmetric case
    row_ptr = np.array([0, 2, 3])
    col_idx = np.array([0, 2, 1])
    vals = np.array([1.0, -2.0, 4.0], dtype=np.float32)
    B = np.array([[1, 10], [2, 20], [3, 30]], dtype=np.float32)
    C, S = oracle.spmm(2, 3, row_ptr, col_idx, vals, "f32", B)
    assert np.array_equal(C, [[1 - 6, 10 - 60], [8, 80]])
    assert np.array_equal(S, [[1 + 6, 10 + 60], [8, 80]])
