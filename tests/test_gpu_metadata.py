"""Bit-exact checks of the GPU-built scheduling metadata against the integer oracle."""
import numpy as np
import pytest

import oracle
import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, make_workload
from dfgnn_synth.workloads import make_graph

pytestmark = pytest.mark.gpu


def default_params(E):
    """Defaults documented in include/dfgnn.h."""
    c = 128
    while c < 512 and c * 16384 < E:
        c *= 2
    return 2 * c, c


def check_metadata(graph, T, C):
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(T, C))
    if C == 0:
        C = default_params(graph.nnz)[1]
    if T == 0:
        T = 2 * C
    assert g.query("n_super_threshold") == T and g.query("n_chunk_edges") == C
    csc = oracle.csc_transpose(graph.indptr, graph.indices)
    rows = oracle.schedule(graph.indptr, T, C)
    cols = oracle.schedule(csc["t_indptr"], T, C)
    get = lambda name: g.query(name).cpu().numpy() if not name.startswith("n_") else g.query(name)
    np.testing.assert_array_equal(get("t_indptr"), csc["t_indptr"])
    np.testing.assert_array_equal(get("t_eid"), csc["t_eid"])
    np.testing.assert_array_equal(get("t_indices"), csc["t_indices"])
    assert get("n_super_rows") == rows["n_super"] and get("n_super_cols") == cols["n_super"]
    np.testing.assert_array_equal(get("row_order"), rows["order"])
    np.testing.assert_array_equal(get("col_order"), cols["order"])
    if rows["n_super"]:
        np.testing.assert_array_equal(get("row_chunk_ptr"), rows["chunk_ptr"])
        np.testing.assert_array_equal(get("row_chunks").reshape(-1, 3), rows["chunks"])
    else:
        assert get("row_chunks").size == 0
    if cols["n_super"]:
        np.testing.assert_array_equal(get("col_chunk_ptr"), cols["chunk_ptr"])
        np.testing.assert_array_equal(get("col_chunks").reshape(-1, 3), cols["chunks"])
    g.close()


@pytest.mark.parametrize("kind", ["random", "hub", "dups", "unsorted", "empty", "chain", "selfloop"])
@pytest.mark.parametrize("T,C", [(4, 3), (8, 8), (1024, 512)])
def test_tiny_graphs(kind, T, C):
    check_metadata(tiny_graph(kind, seed=5, n=40), T, C)


@pytest.mark.parametrize("name,shrink,T,C", [("cfg1", 1, 32, 16), ("cfg2", 1, 16, 8), ("cfg3", 1, 256, 100),
                                             ("cfg3", 1, 0, 0), ("cfg4", 4, 1024, 512), ("cfg5", 64, 64, 64)])
def test_workload_graphs(name, shrink, T, C):
    # spans many sort tiles (4096 keys) with a ragged tail and several radix passes
    check_metadata(make_graph(make_workload(name, shrink=shrink)), T, C)


def test_graph_from_an_unsorted_edge_list():
    """from_edge_index groups edges by destination (stable) and returns the permutation to CSR order."""
    import torch
    from dfgnn_synth import from_edge_list
    rng = np.random.default_rng(6)
    n, e = 300, 2500
    src, dst = rng.integers(0, n, e), rng.integers(0, n, e)
    g, perm = dfgnn.Graph.from_edge_index(torch.from_numpy(src), torch.from_numpy(dst), n)
    ref = from_edge_list(n, src, dst, sort=False)
    assert np.array_equal(g.indptr.cpu().numpy(), ref.indptr) and np.array_equal(g.indices.cpu().numpy(), ref.indices)
    p = perm.cpu().numpy()
    assert np.array_equal(src[p], ref.indices) and np.array_equal(dst[p], ref.rows_of_edges())
    with pytest.raises(ValueError):
        dfgnn.Graph.from_edge_index(torch.tensor([0, n]), torch.tensor([1, 2]), n)
    g.close()


def test_graph_from_a_list_of_small_graphs():
    """from_graph_list offsets the node ids of every graph, builds the block-diagonal CSR and announces the
    batch; the layer on the batch equals the layer on every graph alone."""
    import torch
    from dfgnn_synth import from_edge_list
    from paper_2411_16127_amd.autograd import gt_conv
    rng = np.random.default_rng(8)
    graphs, all_src, all_dst, off = [], [], [], 0
    for _ in range(37):
        n = int(rng.integers(3, 30))
        pairs = np.unique(rng.integers(0, n, size=(4 * n, 2)), axis=0)  # no repeated edge
        graphs.append((torch.from_numpy(pairs[:, 0]), torch.from_numpy(pairs[:, 1]), n))
        all_src.append(pairs[:, 0] + off); all_dst.append(pairs[:, 1] + off)
        off += n
    g, perm, bp = dfgnn.Graph.from_graph_list(graphs)
    ref = from_edge_list(off, np.concatenate(all_src), np.concatenate(all_dst), sort=False)
    assert np.array_equal(g.indptr.cpu().numpy(), ref.indptr) and np.array_equal(g.indices.cpu().numpy(), ref.indices)
    assert np.array_equal(bp.cpu().numpy(), np.cumsum([0] + [n for _, _, n in graphs]))
    assert np.array_equal(np.concatenate(all_src)[perm.cpu().numpy()], ref.indices)
    assert g.query("n_batch_dense") == 1 and g.query("n_xcd_group") == 32
    gen = torch.Generator(device="cuda").manual_seed(3)
    q, k, v = (torch.randn((off, 2, 16), device="cuda", generator=gen) for _ in range(3))
    whole = gt_conv(g, q, k, v)
    for b in (0, 17, 36):
        lo, hi = int(bp[b]), int(bp[b + 1])
        single, _ = dfgnn.Graph.from_edge_index(graphs[b][0], graphs[b][1], graphs[b][2])
        alone = gt_conv(single, q[lo:hi].contiguous(), k[lo:hi].contiguous(), v[lo:hi].contiguous())
        torch.testing.assert_close(whole[lo:hi], alone, rtol=1e-4, atol=1e-5)
        single.close()
    with pytest.raises(ValueError):
        dfgnn.Graph.from_graph_list([(torch.tensor([0, 3]), torch.tensor([1, 1]), 3)])
    g.close()
