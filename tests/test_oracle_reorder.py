"""Pins of the preprocessing oracle (Section IV-A: Reverse Cuthill-McKee reordering, Matrix Market input):
closed forms, hand-written fixtures and structural invariants -- nothing here calls the GPU library."""
import os

import numpy as np
import pytest

from oracle import reorder
from reorder_checks import assert_valid_rcm

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _csr_from_edges(m, edges, symmetric=True, diagonal=False):
    d = np.zeros((m, m), bool)
    for i, j in edges:
        d[i, j] = True
        if symmetric:
            d[j, i] = True
    if diagonal:
        d[np.arange(m), np.arange(m)] = True
    rp = np.concatenate([[0], np.cumsum(d.sum(1))]).astype(np.int32)
    ci = np.nonzero(d)[1].astype(np.int32)
    return rp, ci


def _scramble(m, edges, seed):
    p = np.random.default_rng(seed).permutation(m)
    return [(int(p[i]), int(p[j])) for i, j in edges]


def _bandwidth_after(m, rp, ci, perm):
    va = np.ones(len(ci), np.float32)
    rp2, ci2, _ = reorder.permute_csr(m, m, rp, ci, va, perm, perm)
    return reorder.bandwidth(m, rp2, ci2)


@pytest.mark.parametrize("m", [2, 9, 40])
def test_rcm_restores_a_scrambled_path_to_bandwidth_one(m):
    # a path has a unique Cuthill-McKee order up to its direction: consecutive numbering
    rp, ci = _csr_from_edges(m, _scramble(m, [(i, i + 1) for i in range(m - 1)], seed=m))
    perm = reorder.rcm(m, rp, ci)
    assert _bandwidth_after(m, rp, ci, perm) == 1
    assert_valid_rcm(m, *reorder.sym_adjacency(m, rp, ci), perm)


def test_rcm_on_a_cycle_star_and_grid():
    m = 12   # cycle: breadth-first numbering from any node alternates sides -> bandwidth 2
    rp, ci = _csr_from_edges(m, _scramble(m, [(i, (i + 1) % m) for i in range(m)], seed=1))
    assert _bandwidth_after(m, rp, ci, reorder.rcm(m, rp, ci)) == 2
    m = 9    # star: a leaf first, then the centre, then the other leaves -> the centre sits next to one end
    rp, ci = _csr_from_edges(m, [(4, j) for j in range(m) if j != 4])
    perm = reorder.rcm(m, rp, ci)
    assert perm[1] == 4 or perm[m - 2] == 4
    assert_valid_rcm(m, *reorder.sym_adjacency(m, rp, ci), perm)
    n = 7    # n x n grid graph: level sets are anti-diagonals of at most n nodes -> bandwidth <= 2n - 1, and >= n
    idx = lambda r, c: r * n + c
    edges = [(idx(r, c), idx(r, c + 1)) for r in range(n) for c in range(n - 1)] + \
            [(idx(r, c), idx(r + 1, c)) for r in range(n - 1) for c in range(n)]
    rp, ci = _csr_from_edges(n * n, _scramble(n * n, edges, seed=2))
    perm = reorder.rcm(n * n, rp, ci)
    assert n <= _bandwidth_after(n * n, rp, ci, perm) <= 2 * n - 1
    assert_valid_rcm(n * n, *reorder.sym_adjacency(n * n, rp, ci), perm)


def test_rcm_uses_the_structure_of_a_plus_a_transpose_and_keeps_components_together():
    # one-directional entries only (strictly upper triangle), two components and an isolated node, with a diagonal
    m = 11
    edges = [(0, 3), (3, 7), (7, 9), (1, 2), (2, 5), (5, 8), (8, 10), (1, 10)]   # node 4 and node 6 are alone
    rp, ci = _csr_from_edges(m, edges, symmetric=False, diagonal=True)
    perm = reorder.rcm(m, rp, ci)
    indptr, indices = reorder.sym_adjacency(m, rp, ci)
    assert_valid_rcm(m, indptr, indices, perm, reorder.degrees(m, rp, ci))
    comp = {0: 0, 3: 0, 7: 0, 9: 0, 1: 1, 2: 1, 5: 1, 8: 1, 10: 1, 4: 2, 6: 3}
    labels = [comp[int(v)] for v in perm]
    assert sum(labels[i] != labels[i + 1] for i in range(m - 1)) == 3          # four contiguous runs
    assert _bandwidth_after(m, rp, ci, perm) <= 2


def test_rcm_on_random_banded_structure_recovers_a_narrow_band():
    rng = np.random.default_rng(5)
    m, hb = 300, 4
    edges = [(i, j) for i in range(m) for j in range(i + 1, min(m, i + hb + 1)) if rng.random() < 0.7]
    rp, ci = _csr_from_edges(m, _scramble(m, edges, seed=6))
    assert reorder.bandwidth(m, rp, ci) > 100
    perm = reorder.rcm(m, rp, ci)
    assert _bandwidth_after(m, rp, ci, perm) <= 3 * hb
    assert_valid_rcm(m, *reorder.sym_adjacency(m, rp, ci), perm)


def test_degree_key_counts_a_stored_diagonal_twice():
    # nodes 0-1-2 in a path, node 1 with a diagonal entry; node 3 alone with a diagonal entry; node 4 alone
    rp, ci = _csr_from_edges(5, [(0, 1), (1, 2), (1, 1), (3, 3)])
    assert reorder.degrees(5, rp, ci).tolist() == [1, 4, 1, 2, 0]
    # the key decides the order: mixed diagonals, random structure -- scipy's order is valid under this key
    rng = np.random.default_rng(9)
    m = 200
    edges = [(int(i), int(j)) for i, j in rng.integers(0, m, size=(500, 2))]
    rp, ci = _csr_from_edges(m, edges)
    assert 0 < np.count_nonzero(np.diff(rp) != reorder.degrees(m, rp, ci)) < m
    assert_valid_rcm(m, *reorder.sym_adjacency(m, rp, ci), reorder.rcm(m, rp, ci), reorder.degrees(m, rp, ci))


def test_permute_csr_matches_dense_indexing():
    rng = np.random.default_rng(7)
    m, k = 13, 17
    dense = np.where(rng.random((m, k)) < 0.3, rng.standard_normal((m, k)), 0).astype(np.float32)
    rp = np.concatenate([[0], np.cumsum((dense != 0).sum(1))]).astype(np.int32)
    ci = np.nonzero(dense)[1].astype(np.int32)
    va = dense[dense != 0]
    rperm, cperm = rng.permutation(m), rng.permutation(k)
    for cp, want in ((cperm, dense[rperm][:, cperm]), (None, dense[rperm])):
        rp2, ci2, va2 = reorder.permute_csr(m, k, rp, ci, va, rperm, cp)
        got = np.zeros((m, k), np.float32)
        for i in range(m):
            assert (np.diff(ci2[rp2[i]:rp2[i + 1]]) > 0).all()
            got[i, ci2[rp2[i]:rp2[i + 1]]] = va2[rp2[i]:rp2[i + 1]]
        assert np.array_equal(got, want)


def test_read_mtx_fixtures():
    m, k, rp, ci, va = reorder.read_mtx(os.path.join(GOLDEN, "general_real_4x5.mtx"))
    assert (m, k) == (4, 5)
    assert rp.tolist() == [0, 3, 4, 6, 7]                       # the explicit zero at (2,2) stays stored
    assert ci.tolist() == [0, 3, 4, 1, 0, 2, 4]
    assert va.tolist() == [1.0, 0.5, -1.0, 0.0, -2.5, 1.5, 7.0]  # 1.25 + 0.25 summed
    m, k, rp, ci, va = reorder.read_mtx(os.path.join(GOLDEN, "symmetric_pattern_5x5.mtx"))
    dense = np.zeros((5, 5))
    for i in range(5):
        dense[i, ci[rp[i]:rp[i + 1]]] = va[rp[i]:rp[i + 1]]
    want = np.zeros((5, 5))
    for i, j in ((0, 0), (2, 0), (3, 1), (4, 2), (4, 4)):
        want[i, j] = want[j, i] = 1
    assert np.array_equal(dense, want) and len(ci) == 8
    m, k, rp, ci, va = reorder.read_mtx(os.path.join(GOLDEN, "skew_integer_3x3.mtx"))
    assert rp.tolist() == [0, 1, 3, 4] and ci.tolist() == [1, 0, 2, 1] and va.tolist() == [-4.0, 4.0, 6.0, -6.0]
