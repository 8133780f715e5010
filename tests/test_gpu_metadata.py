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


def check_metadata(graph, T, C, batch_ptr=None, flags=0):
    """batch_ptr: build through dfgnn_graph_create_batch (metadata and batch structure in one call)."""
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(T, C, flags), batch_ptr=batch_ptr)
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


def block_diagonal(sizes, density, seed, shuffle_rows=False, repeats=False):
    """Batch of random graphs of the given node counts (zero allowed); optionally with the sources of every
    row in random order and with repeated edges."""
    from dfgnn_synth import from_edge_list
    rng = np.random.default_rng(seed)
    bp = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    src, dst = [], []
    for b, n in enumerate(sizes):
        if n == 0:
            continue
        adj = rng.random((n, n)) < density
        d, s_ = np.nonzero(adj)
        if repeats and d.size:
            extra = rng.integers(0, d.size, d.size // 4)
            d, s_ = np.concatenate([d, d[extra]]), np.concatenate([s_, s_[extra]])
        if shuffle_rows:
            perm = rng.permutation(d.size)
            d, s_ = d[perm], s_[perm]
        src.append(s_ + bp[b]); dst.append(d + bp[b])
    src = np.concatenate(src) if src else np.empty(0, np.int64)
    dst = np.concatenate(dst) if dst else np.empty(0, np.int64)
    return from_edge_list(int(bp[-1]), src, dst, sort=not shuffle_rows, batch_ptr=bp)


# one workgroup per graph: one radix pass up to 64 nodes, two above; empty graphs; a graph that is too large
# for a segment sends the whole batch through the general builder; T and C small enough for super rows
@pytest.mark.parametrize("sizes,density,T,C", [
    ([5, 1, 17, 64, 0, 33], 0.4, 1024, 512), ([65, 130, 3, 700], 0.1, 16, 8), ([0, 0, 9], 0.5, 4, 3),
    ([4096, 10], 0.002, 64, 32), ([4097, 10], 0.002, 64, 32), ([40] * 300, 0.3, 0, 0), ([1] * 70, 1.0, 0, 0),
    # 300 x 300 edges exceed a segment, 254 x 254 do not: some graphs are processed, one is refused, and the
    # whole batch goes through the general builder (the refused graph's counts must not be used by the others)
    ([254, 20, 300, 254, 7], 1.0, 0, 0)])
@pytest.mark.parametrize("messy", [False, True])
def test_batches_in_one_call(sizes, density, T, C, messy):
    graph = block_diagonal(sizes, density, seed=len(sizes), shuffle_rows=messy, repeats=messy)
    check_metadata(graph, T, C, batch_ptr=graph.batch_ptr)


def test_batch_tables_of_the_one_call_route_equal_those_of_the_two_calls():
    """Tile tables and adjacency bit masks (what the dense-tile kernels read) from dfgnn_graph_create_batch
    against dfgnn_graph_create + dfgnn_graph_set_batch, byte for byte."""
    import torch
    graph = block_diagonal([30, 64, 65, 7, 512, 100, 0, 16], 0.2, seed=3)
    one = dfgnn.Graph(graph.indptr, graph.indices, None, batch_ptr=graph.batch_ptr)
    two = dfgnn.Graph(graph.indptr, graph.indices, None)
    bp = torch.as_tensor(graph.batch_ptr, dtype=torch.int32).cuda()
    n_graphs = bp.numel() - 1
    nbytes = dfgnn.graph_batch_bytes(graph.n, n_graphs)
    buf = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dfgnn.graph_set_batch(two.handle, bp, n_graphs, buf, nbytes)
    assert one.query("n_batch_dense") == 1 == two.query("n_batch_dense")
    words = 8  # the largest graph has 512 nodes
    mask_bytes = graph.n * words * 8
    tiles = sum((n + 15) // 16 for n in [30, 64, 65, 7, 512, 100, 0, 16])
    align = lambda x: (x + 255) // 256 * 256
    full = align(graph.n * 8 * 8)  # the layout reserves masks of 8 words per node
    a, b = one.batch_meta.cpu().numpy(), buf.cpu().numpy()
    assert np.array_equal(a[:mask_bytes], b[:mask_bytes])                          # row masks
    assert np.array_equal(a[full:full + mask_bytes], b[full:full + mask_bytes])    # column masks
    off = 2 * full
    assert np.array_equal(a[off:off + 4 * (n_graphs + 1)], b[off:off + 4 * (n_graphs + 1)])  # tile pointer
    off += align(4 * (n_graphs + 2))
    assert np.array_equal(a[off:off + 4 * tiles], b[off:off + 4 * tiles])          # graph of every tile
    one.close(); two.close()


def test_batch_errors_in_one_call():
    import torch
    graph = block_diagonal([10, 12, 9], 0.5, seed=1)
    bad_ptr = graph.batch_ptr.copy(); bad_ptr[1] = 25  # decreasing afterwards
    with pytest.raises(dfgnn.DfgnnError) as e:
        dfgnn.Graph(graph.indptr, graph.indices, None, batch_ptr=bad_ptr)
    assert e.value.status == 1 and "batch_ptr" in str(e.value)
    cross = graph.indices.copy(); cross[0] = 30  # row 0 (first graph) reads a node of the last graph
    with pytest.raises(dfgnn.DfgnnError) as e:
        dfgnn.Graph(graph.indptr, cross, None, batch_ptr=graph.batch_ptr)
    assert e.value.status == 1 and "different graphs" in str(e.value)
    out_of_range = graph.indices.copy(); out_of_range[5] = graph.n
    with pytest.raises(dfgnn.DfgnnError) as e:
        dfgnn.Graph(graph.indptr, out_of_range, None, batch_ptr=graph.batch_ptr)
    assert e.value.status == 1 and "malformed CSR" in str(e.value)
    wrong_end = graph.indptr.copy(); wrong_end[-1] -= 1
    for kw in ({}, {"batch_ptr": graph.batch_ptr}):  # the small-graph route of dfgnn_graph_create reports the same
        with pytest.raises(dfgnn.DfgnnError) as e:
            dfgnn.Graph(wrong_end, graph.indices, None, **kw)  # indptr[N] != E
        assert e.value.status == 1 and "malformed CSR" in str(e.value)


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
