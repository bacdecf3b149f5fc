"""Property checks for Cuthill-McKee orderings, shared by the oracle's pins and the library's parity tests.

Several orderings are valid (ties between nodes of equal degree may be broken either way), so what is checked
is what every valid one has: the reverse of the permutation is a breadth-first order in which each component
starts at an unvisited node of least degree and every node's not-yet-numbered neighbours follow as one run in
order of non-decreasing degree.
"""
import numpy as np


def assert_valid_rcm(m, indptr, indices, perm, deg=None):
    """indptr/indices: neighbour lists of the structure of A + A^T; perm[new] = old; deg: the ordering key of
    every node (default: its number of neighbours)."""
    perm = np.asarray(perm, dtype=np.int64)
    assert perm.shape == (m,) and np.array_equal(np.sort(perm), np.arange(m)), "not a permutation"
    order = perm[::-1]
    deg = np.diff(indptr) if deg is None else np.asarray(deg)
    visited = np.zeros(m, bool)
    pos = 0
    for i in range(m):
        if i == pos:  # the queue ran empty: a new component starts
            seed = order[pos]
            assert not visited[seed]
            assert deg[seed] == deg[~visited].min(), "component does not start at a node of least degree"
            visited[seed] = True
            pos += 1
        node = order[i]
        nb = np.unique(indices[indptr[node]:indptr[node + 1]])
        nb = nb[~visited[nb]]
        block = order[pos:pos + len(nb)]
        assert np.array_equal(np.sort(block), nb), "neighbours of node %d are not numbered next" % node
        assert (np.diff(deg[block]) >= 0).all(), "neighbours of node %d are not in order of degree" % node
        visited[block] = True
        pos += len(nb)
    assert pos == m
