"""Pins for the integer metadata oracle: brute force on tiny graphs and structural invariants."""
import numpy as np
import pytest

import oracle
from dfgnn_synth import tiny_graph, make_workload
from dfgnn_synth.workloads import make_graph


@pytest.mark.parametrize("kind", ["random", "hub", "dups", "unsorted", "empty", "chain", "selfloop"])
def test_csc_against_brute_force(kind):
    g = tiny_graph(kind, seed=1, n=20)
    t = oracle.csc_transpose(g.indptr, g.indices)
    rows = g.rows_of_edges()
    pos = 0
    for j in range(g.n):  # O(N*E): scan all edges for every column, in CSR order
        assert t["t_indptr"][j] == pos
        for e in range(g.nnz):
            if g.indices[e] == j:
                assert t["t_eid"][pos] == e and t["t_indices"][pos] == rows[e]
                pos += 1
    assert t["t_indptr"][g.n] == pos == g.nnz


def test_transpose_twice_is_identity():
    g = make_graph(make_workload("cfg1"))
    t = oracle.csc_transpose(g.indptr, g.indices)
    tt = oracle.csc_transpose(t["t_indptr"], t["t_indices"])
    np.testing.assert_array_equal(tt["t_indptr"], g.indptr)
    np.testing.assert_array_equal(tt["t_indices"], g.indices)  # sources ascending in a row, so order is recovered
    np.testing.assert_array_equal(t["t_eid"][tt["t_eid"]], np.arange(g.nnz))


@pytest.mark.parametrize("T,C", [(8, 4), (16, 16), (5, 7), (1000, 64)])
def test_schedule_structure(T, C):
    g = tiny_graph("hub", seed=3, n=40)
    deg = g.degrees()
    s = oracle.schedule(g.indptr, T, C)
    order = s["order"]
    assert sorted(order.tolist()) == list(range(g.n))
    ns = s["n_super"]
    sup, rest = order[:ns], order[ns:]
    assert np.all(deg[sup] >= T) and np.all(deg[rest] < T)
    assert np.all(np.diff(sup) > 0)
    bl = np.array([int(d).bit_length() for d in deg[rest]])
    assert np.all(np.diff(bl) <= 0)  # longer rows first
    for b in np.unique(bl):
        assert np.all(np.diff(rest[bl == b]) > 0)  # stable inside a bucket
    # chunks tile every super row exactly once, in order, with sizes <= C
    cp, ch = s["chunk_ptr"], s["chunks"]
    assert cp[0] == 0 and cp[-1] == len(ch)
    for k, row in enumerate(sup):
        mine = ch[cp[k]:cp[k + 1]]
        assert np.all(mine[:, 0] == row)
        assert mine[0, 1] == g.indptr[row] and mine[-1, 2] == g.indptr[row + 1]
        assert np.all(mine[1:, 1] == mine[:-1, 2])
        sizes = mine[:, 2] - mine[:, 1]
        assert np.all(sizes > 0) and np.all(sizes <= C) and np.all(sizes[:-1] == C)


def test_bucket_key_hand_example():
    # degrees 0,1,2,3,4,9 ; T = 9 -> row 5 is super; keys: 33,32,31,31,30,0
    indptr = np.array([0, 0, 1, 3, 6, 10, 19])
    s = oracle.schedule(indptr, 9, 4)
    assert s["order"].tolist() == [5, 4, 2, 3, 1, 0]
    assert s["n_super"] == 1
    assert s["chunks"].tolist() == [[5, 10, 14], [5, 14, 18], [5, 18, 19]]
