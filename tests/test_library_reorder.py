"""The library's host-side preprocessing (Reverse Cuthill-McKee, CSR permutation, Matrix Market reader) against
the oracle.  Orderings: several are valid (ties), so validity and quality are compared, not the permutations;
permuted arrays and file contents must be bit-exact.  No GPU is needed here."""
import os

import numpy as np
import pytest

from oracle import reorder
from paper_2604_17834_amd import binding as asp
from paper_2604_17834_amd import synth
from reorder_checks import assert_valid_rcm

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _square_structures():
    rng = np.random.default_rng(21)
    out = []
    # scrambled band, scrambled grid, random unsymmetric structure with isolated nodes, zipf graph, empty matrix
    m = 400
    p = rng.permutation(m)
    keys = sorted({(int(p[i]), int(p[j])) for i in range(m) for j in range(max(0, i - 5), min(m, i + 6)) if rng.random() < 0.6})
    out.append((m, keys))
    n = 15
    p = rng.permutation(n * n)
    keys = set()
    for r in range(n):
        for c in range(n):
            for rr, cc in ((r, c + 1), (r + 1, c)):
                if rr < n and cc < n:
                    keys.add((int(p[r * n + c]), int(p[rr * n + cc])))
                    keys.add((int(p[rr * n + cc]), int(p[r * n + c])))
    out.append((n * n, sorted(keys)))
    a = synth.random_csr(300, 300, 0.004, seed=22, dtype="f32", empty_row_frac=0.3)
    out.append((a.m, None, a))
    a = synth.zipf_graph(2000, 2000, 6 * 2000, seed=23, cap=300)
    out.append((a.m, None, a))
    out.append((50, []))
    res = []
    for item in out:
        if len(item) == 3:
            res.append((item[0], item[2].row_ptr, item[2].col_idx))
        else:
            m, keys = item
            rows = np.array([k[0] for k in keys], dtype=np.int64)
            rp = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=m))]).astype(np.int32) if keys else np.zeros(m + 1, np.int32)
            res.append((m, rp, np.array([k[1] for k in keys], dtype=np.int32)))
    return res


@pytest.mark.parametrize("case", range(5))
def test_rcm_is_a_valid_ordering_and_as_narrow_as_the_oracles(case):
    m, rp, ci = _square_structures()[case]
    perm = asp.asp_rcm(m, rp, ci)
    indptr, indices = reorder.sym_adjacency(m, rp, ci)
    deg = reorder.degrees(m, rp, ci)
    assert_valid_rcm(m, indptr, indices, perm, deg)
    va = np.ones(len(ci), np.float32)
    bw = lambda q: reorder.bandwidth(m, *reorder.permute_csr(m, m, rp, ci, va, q, q)[:2])
    ours, theirs = bw(perm), bw(reorder.rcm(m, rp, ci))
    assert_valid_rcm(m, indptr, indices, reorder.rcm(m, rp, ci), deg)
    # both are Cuthill-McKee orders from least-degree start nodes; tie-breaking may differ, quality may not much
    assert ours <= max(theirs + 2, int(1.25 * theirs)), (ours, theirs)
    if case == 0:
        assert ours <= 15 and reorder.bandwidth(m, rp, ci) > 200
    assert np.array_equal(perm, asp.asp_rcm(m, rp, ci))   # deterministic


def test_rcm_path_and_errors():
    m = 30
    p = np.random.default_rng(3).permutation(m)
    keys = sorted([(int(p[i]), int(p[i + 1])) for i in range(m - 1)])
    rows = np.array([k[0] for k in keys])
    rp = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=m))]).astype(np.int32)
    ci = np.array([k[1] for k in keys], np.int32)
    perm = asp.asp_rcm(m, rp, ci)
    va = np.ones(len(ci), np.float32)
    assert reorder.bandwidth(m, *reorder.permute_csr(m, m, rp, ci, va, perm, perm)[:2]) == 1
    L = asp.lib()
    out = np.zeros(m, np.int32)
    assert L.asp_rcm(m, None, ci.ctypes.data, out.ctypes.data) == asp.ASP_ERR_INVALID_ARG
    assert L.asp_rcm(0, rp.ctypes.data, ci.ctypes.data, out.ctypes.data) == asp.ASP_ERR_INVALID_ARG
    bad = ci.copy()
    bad[0] = m    # column outside the square matrix
    assert L.asp_rcm(m, rp.ctypes.data, bad.ctypes.data, out.ctypes.data) == asp.ASP_ERR_INVALID_CSR


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_permute_csr_bit_exact_vs_oracle(dtype):
    a = synth.random_csr(123, 77, 0.08, seed=31, dtype=dtype, empty_row_frac=0.2, dist="normal")
    rng = np.random.default_rng(32)
    rperm, cperm = rng.permutation(a.m), rng.permutation(a.k)
    for cp in (cperm, None):
        want = reorder.permute_csr(a.m, a.k, a.row_ptr, a.col_idx, a.values, rperm, cp)
        got = asp.asp_permute_csr(a.m, a.k, a.row_ptr, a.col_idx, a.values, dtype, rperm, cp)
        for g, w in zip(got, want):
            assert g.dtype == w.dtype and np.array_equal(g, w)
    notperm = rperm.copy()
    notperm[0] = notperm[1]
    assert asp.asp_permute_csr(a.m, a.k, a.row_ptr, a.col_idx, a.values, dtype, notperm, None, check=False) == asp.ASP_ERR_INVALID_ARG
    assert asp.asp_permute_csr(a.m, a.k, a.row_ptr, a.col_idx, a.values, dtype, rperm, rperm[:a.k] * 0, check=False) == asp.ASP_ERR_INVALID_ARG


def test_symmetric_permutation_commutes_with_the_product():
    # (P A P^T)(P B) = P (A B): reordering changes the layout, never the result (fp64 oracle on both sides)
    import oracle
    a = synth.zipf_graph(512, 512, 8 * 512, seed=41, cap=100)
    perm = asp.asp_rcm(a.m, a.row_ptr, a.col_idx)
    rp, ci, va = asp.asp_permute_csr(a.m, a.k, a.row_ptr, a.col_idx, a.values, "f32", perm, perm)
    B = synth.dense_normal(a.k, 8, "f32", seed=42)
    c0, _ = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, "f32", B, want_bound=False)
    c1, _ = oracle.spmm(a.m, a.k, rp, ci, va, "f32", np.ascontiguousarray(B[perm]), want_bound=False)
    assert np.allclose(c1, c0[perm], rtol=0, atol=1e-12)


@pytest.mark.parametrize("name", ["general_real_4x5.mtx", "symmetric_pattern_5x5.mtx", "skew_integer_3x3.mtx"])
def test_mtx_reader_bit_exact_vs_oracle_on_fixtures(name):
    path = os.path.join(GOLDEN, name)
    want = reorder.read_mtx(path)
    got = asp.asp_mtx_read(path)
    assert got[:2] == want[:2]
    for g, w in zip(got[2:], want[2:]):
        assert g.dtype == w.dtype and np.array_equal(g, w)


def test_mtx_reader_on_a_generated_file_and_errors(tmp_path):
    a = synth.random_csr(60, 45, 0.1, seed=51, dtype="f32", dist="normal")
    rows = np.repeat(np.arange(a.m), np.diff(a.row_ptr))
    order = np.random.default_rng(52).permutation(a.nnz)
    p = tmp_path / "gen.mtx"
    with open(p, "w") as f:
        f.write("%%%%MatrixMarket matrix coordinate real general\n%% generated\n\n%d %d %d\n" % (a.m, a.k, a.nnz))
        for t in order:
            f.write("%d %d %.9g\n" % (rows[t] + 1, a.col_idx[t] + 1, a.values[t]))
    m, k, rp, ci, va = asp.asp_mtx_read(str(p))
    assert (m, k) == (a.m, a.k) and np.array_equal(rp, a.row_ptr) and np.array_equal(ci, a.col_idx)
    assert np.array_equal(va, a.values)            # %.9g round-trips a float32
    want = reorder.read_mtx(str(p))
    assert np.array_equal(va, want[4]) and np.array_equal(ci, want[3])

    def status(text):
        q = tmp_path / "bad.mtx"
        q.write_text(text)
        return asp.asp_mtx_read(str(q), check=False)
    assert asp.asp_mtx_read(str(tmp_path / "missing.mtx"), check=False) == asp.ASP_ERR_INVALID_ARG
    assert status("hello\n1 1 1\n") == asp.ASP_ERR_INVALID_CSR
    assert status("%%MatrixMarket matrix array real general\n2 2\n1\n2\n3\n4\n") == asp.ASP_ERR_UNSUPPORTED
    assert status("%%MatrixMarket matrix coordinate complex general\n1 1 1\n1 1 1 0\n") == asp.ASP_ERR_UNSUPPORTED
    assert status("%%MatrixMarket matrix coordinate real general\n2 2 1\n3 1 1.0\n") == asp.ASP_ERR_INVALID_CSR
    assert status("%%MatrixMarket matrix coordinate real general\n2 2 2\n1 1 1.0\n") == asp.ASP_ERR_INVALID_CSR
    assert "ends after" in asp.asp_last_error()
