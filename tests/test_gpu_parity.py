"""Element-by-element parity of the HIP path (through the C ABI) with the CPU oracle."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, complete_graph, make_workload, make_features
from dfgnn_synth.workloads import make_graph, Workload
from gpu_harness import run_gpu, run_oracle, compare_all

pytestmark = pytest.mark.gpu


def small_workload(model, H, D, dtype="f32"):
    scale = {"gt": 1.0 / np.sqrt(D), "gat": 1.0, "agnn": 1.3}[model]
    return Workload("tiny", 90, model, H, D, dtype, float(scale))


# (H, D) pairs: the compile-time geometries of the benchmark shapes and several run-time ones,
# including a head count that leaves padded lanes (H=3)
SHAPES_F32 = [(1, 64), (8, 16), (8, 8), (2, 4), (3, 8), (1, 16), (4, 32), (1, 256), (2, 128)]
SHAPES_BF16 = [(8, 16), (1, 8), (3, 16), (2, 64), (1, 512)]


@pytest.mark.parametrize("model", ["gt", "gat", "agnn"])
@pytest.mark.parametrize("H,D", SHAPES_F32)
@pytest.mark.parametrize("kind", ["random", "hub", "dups", "unsorted", "empty", "selfloop"])
def test_tiny_graphs_f32(model, H, D, kind):
    graph = tiny_graph(kind, seed=2, n=70)
    w = small_workload(model, H, D)
    feats = make_features(w, graph.n)
    # threshold 8 / chunk 5: hub rows and columns go through the chunk + merge path with ragged chunks
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


@pytest.mark.parametrize("model", ["gt", "gat", "agnn"])
@pytest.mark.parametrize("H,D", SHAPES_BF16)
def test_tiny_graphs_bf16(model, H, D):
    graph = tiny_graph("hub", seed=3, n=70)
    w = small_workload(model, H, D, "bf16")
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("H,D", SHAPES_BF16)
@pytest.mark.parametrize("kind", ["hub", "chain", "empty"])
def test_tiny_graphs_f16(model, H, D, kind):
    graph = tiny_graph(kind, seed=3, n=70)
    w = Workload("tiny", 92, model, H, D, "f16", {"gt": float(1.0 / np.sqrt(D)), "agnn": 1.3}.get(model, 1.0))
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


# rows of 64 or 128 features split into 1 to 16 heads: every lane geometry with compile-time head reductions
FULL_ROW_SHAPES = [("f32", H, 64 // H) for H in (1, 2, 4, 8)] + [("f32", H, 128 // H) for H in (1, 2, 4, 8, 16)] + \
                  [("bf16", H, 128 // H) for H in (1, 2, 4, 8, 16)] + [("bf16", H, 64 // H) for H in (1, 2, 4, 8)] + \
                  [("f16", H, 128 // H) for H in (1, 2, 4, 8, 16)] + [("f16", H, 64 // H) for H in (1, 2, 4, 8)]


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("dtype,H,D", FULL_ROW_SHAPES)
def test_full_row_geometries(model, dtype, H, D):
    graph = tiny_graph("hub", seed=11, n=90)
    w = Workload("tiny", 99, model, H, D, dtype, {"gt": float(1.0 / np.sqrt(D)), "agnn": 1.3}.get(model, 1.0))
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


# rows wider than one wavefront of 16-byte lanes: the layer runs in groups of heads
WIDE_SHAPES = [("f32", 8, 64), ("f32", 3, 128), ("f32", 2, 256), ("f32", 16, 32), ("bf16", 16, 64), ("bf16", 3, 256),
               ("f32", 5, 64), ("f16", 16, 64)]


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("dtype,H,D", WIDE_SHAPES)
def test_rows_wider_than_a_wavefront(model, dtype, H, D):
    graph = tiny_graph("hub", seed=13, n=60)
    w = Workload("tiny", 100, model, H, D, dtype, {"gt": float(1.0 / np.sqrt(D)), "agnn": 1.3}.get(model, 1.0))
    feats = make_features(w, graph.n)
    if model == "gt":  # with an edge term too: its head offset moves with the group
        rng = np.random.default_rng(5)
        feats["edge_bias"] = rng.standard_normal((graph.nnz, H)).astype(np.float32)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


@pytest.mark.parametrize("model", ["gt", "gat", "agnn"])
def test_complete_graph(model):
    graph = complete_graph(67)  # every row has 67 neighbours: several unrolled rounds plus a ragged tail
    w = small_workload(model, 2, 16)
    feats = make_features(w, graph.n)
    for sched in (None, dfgnn.SchedParams(32, 16)):
        res, g = run_gpu(graph, w, feats, sched)
        compare_all(res, run_oracle(graph, w, feats), w)
        g.close()


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_hub_rows_with_hundreds_of_chunks(model, dtype):
    """16 hub rows of 6,250 neighbours cut into chunks of 16 edges: their 391 partials each are merged in two
    levels (groups of chunks first, then the groups).  The hubs' sources are hub columns too for no node here, so
    the column side is covered by the transposed graph: the same layer on the graph with every edge reversed."""
    from dfgnn_synth import from_edge_list
    base = make_workload("cfg4", shrink=32)
    graph = make_graph(base)
    scale = {"gt": 0.25, "agnn": 1.3}.get(model, 1.0)
    w = Workload("hubs", 93, model, 2, 16, dtype, float(scale))
    for g_in in (graph, from_edge_list(graph.n, graph.rows_of_edges(), graph.indices)):  # hub rows; hub columns
        feats = make_features(w, g_in.n)
        res, g = run_gpu(g_in, w, feats, dfgnn.SchedParams(64, 16))
        assert g.query("n_super_rows") + g.query("n_super_cols") >= 16
        compare_all(res, run_oracle(g_in, w, feats), w)
        g.close()


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_single_edge_row_beside_longer_rows_16_bit(model, dtype):
    """Rows of one edge that share a wavefront with rows of 9 to 11 edges: the longer rows take several rounds of
    the edge loop, during which the slot of the single-edge row is idle and must keep what its only edge left
    (the value the column side subtracts to reach an exact zero for that edge's score gradient)."""
    from dfgnn_synth import from_edge_list
    n = 14
    rows, cols = [0, 5], [3, 7]  # two rows with one edge each
    rng = np.random.default_rng(5)
    for i in (1, 2, 4, 6, 9):
        nb = rng.choice(n, size=9 + i % 3, replace=False)
        rows += [i] * len(nb); cols += [int(j) for j in nb]
    graph = from_edge_list(n, np.array(cols, np.int64), np.array(rows, np.int64))  # (sources, destinations = rows)
    scale = {"gt": 0.25, "agnn": 1.3}.get(model, 1.0)
    w = Workload("single_edge_mix", 41, model, 2, 16, dtype, float(scale))
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats)
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


def test_split_rows_match_unsplit_rows():
    """The chunk + merge path and the one-wave-per-row path give the same numbers (to rounding)."""
    graph = make_graph(make_workload("cfg1"))
    w = make_workload("cfg1")
    feats = make_features(w, graph.n)
    a, g1 = run_gpu(graph, w, feats, dfgnn.SchedParams(1 << 30, 1 << 30))
    b, g2 = run_gpu(graph, w, feats, dfgnn.SchedParams(16, 8))
    assert g1.query("n_super_rows") == 0 and g2.query("n_super_rows") > 10
    for key in a:
        np.testing.assert_allclose(a[key], b[key], rtol=2e-5, atol=2e-6)
    g1.close(); g2.close()


def test_backward_as_one_launch_matches_two_launches():
    """Small fp32 GT graphs without super rows run the row side and the column side of the backward pass as one
    launch (the column side recomputes delta from the output rows); flag 64 keeps them apart.  Both match the
    oracle, and each other to rounding."""
    w = make_workload("cfg1")
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    ref = run_oracle(graph, w, feats)
    one, g1 = run_gpu(graph, w, feats)
    two, g2 = run_gpu(graph, w, feats, dfgnn.SchedParams(flags=64))
    assert g1.query("n_super_rows") == 0 and g1.query("n_super_cols") == 0
    compare_all(one, ref, w)
    compare_all(two, ref, w)
    for key in ("d_x",):  # the row side is the same kernel code
        assert np.array_equal(one[key], two[key])
    for key in ("d_k", "d_v"):
        np.testing.assert_allclose(one[key], two[key], rtol=2e-5, atol=2e-6)
    g1.close(); g2.close()


def test_large_scores_are_stable():
    graph = tiny_graph("hub", seed=4, n=70)
    w = small_workload("gt", 1, 64)
    feats = make_features(w, graph.n)
    feats["q"] = feats["q"] * np.float32(40.0)  # scores of order +-500
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    for key, val in res.items():
        assert np.all(np.isfinite(val) | np.isneginf(val)), key
    # a score of magnitude 500 carries an fp32 rounding error of ~3e-5 in the exponent, so the attention
    # weights are only good to ~1e-4 relative; gradients (which cancel) are checked ten times looser
    compare_all(res, run_oracle(graph, w, feats), w, tol=(1e-3, 1e-4, 0.0))
    g.close()


def test_results_are_bitwise_reproducible():
    graph = make_graph(make_workload("cfg3", shrink=16))
    w = make_workload("cfg3", shrink=16)
    feats = make_features(w, graph.n)
    a, g = run_gpu(graph, w, feats, dfgnn.SchedParams(64, 32))
    b, _ = run_gpu(graph, w, feats, g=g)
    for key in a:
        assert np.array_equal(a[key], b[key]), key
    g.close()


# ------------------------------------------------------------------ the five workloads, reduced in size
@pytest.mark.parametrize("name,shrink,T,C", [("cfg1", 1, 0, 0), ("cfg1", 1, 64, 32), ("cfg2", 8, 0, 0),
                                             ("cfg3", 8, 0, 0), ("cfg3", 8, 128, 64), ("cfg4", 16, 0, 0),
                                             ("cfg5", 256, 0, 0), ("cfg5", 256, 96, 40)])
def test_workloads_reduced(name, shrink, T, C):
    w = make_workload(name, shrink=shrink)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(T, C) if T else None)
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


# the large workloads with bf16 node tensors (half the row bytes; feature-dimension study of Appendix C)
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("name,shrink,T,C", [("cfg3", 8, 0, 0), ("cfg3", 8, 128, 64), ("cfg4", 16, 0, 0),
                                             ("cfg5", 256, 0, 0), ("cfg5", 256, 96, 40), ("cfg2", 8, 0, 0)])
def test_workloads_reduced_16_bit(name, shrink, T, C, dtype):
    w = make_workload(name, shrink=shrink, dtype=dtype)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(T, C) if T else None)
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


# ------------------------------------------------------------------ full benchmark sizes
@pytest.mark.parametrize("name,dtype", [("cfg1", None), ("cfg2", None), ("cfg3", None), ("cfg4", None),
                                        ("cfg3", "bf16"), ("cfg4", "bf16"), ("cfg3", "f16"), ("cfg4", "f16")])
def test_workloads_full_size(name, dtype):
    w = make_workload(name, **({"dtype": dtype} if dtype else {}))
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats)  # default scheduling parameters, as the benchmark runs it
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cfg5_full_size_sampled(dtype):
    """123M edges: the oracle evaluates sampled nodes one by one (rows for O / dQ, and every row that a
    sampled node feeds for its dK / dV), the GPU runs the whole graph with the default schedule, as the
    benchmark does.  The sampled columns include super columns (out-degree >= super_threshold), whose dK / dV
    go through the chunk + merge path of the column pass: the column of largest out-degree and the two
    closest to the threshold from above."""
    w = make_workload("cfg5", dtype=dtype)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    print(f"cfg5 {dtype}: graph and features drawn", flush=True)
    res, g = run_gpu(graph, w, feats)
    print("GPU pass done; oracle on the sampled rows and columns", flush=True)
    T = g.query("n_super_threshold")
    deg = graph.degrees()
    rng = np.random.default_rng(77)
    sample = np.unique(np.concatenate([rng.choice(graph.n, 48, replace=False), np.argsort(deg)[-3:],
                                       np.argsort(deg)[:2]]))
    out_deg = np.bincount(graph.indices, minlength=graph.n)
    light = sample[out_deg[sample] < 400]  # columns with few feeding rows
    by_out = np.argsort(out_deg, kind="stable")
    first_super = int(np.searchsorted(out_deg[by_out], T))
    assert g.query("n_super_cols") == graph.n - first_super > 3
    heavy = np.concatenate([by_out[first_super:first_super + 2], by_out[-1:]])  # super columns
    assert np.all(out_deg[heavy] >= T)
    cols = np.union1d(light, heavy)
    rows_of_edges = graph.rows_of_edges()
    feed = np.unique(rows_of_edges[np.isin(graph.indices, cols)])
    ref = run_oracle(graph, w, feats, rows=sample, backward_rows=np.union1d(sample, feed))
    compare_all(res, ref, w, rows=sample, keys=["out", "row_max", "row_sum", "d_x"])
    compare_all(res, ref, w, rows=cols, keys=["d_k", "d_v"])
    g.close()


@pytest.mark.parametrize("N", [8388000, 8390000])
def test_node_tensors_around_4_gib(N):
    """Gathers address node rows with 32-bit byte offsets up to 4 GiB minus one row and with 64-bit addresses
    beyond: a graph whose tensors end 300 KB below 4 GiB (N = 8,388,000 rows of 512 bytes) and one whose
    tensors end 700 KB above (N = 8,390,000), checked on rows and columns at both ends of the node range.
    Tensors are drawn on the GPU; the oracle gets the compact sub-problem of the sampled rows (whole
    neighbourhoods) and of every row that feeds a sampled column."""
    import torch
    from dfgnn_synth import from_edge_list
    H, D = 8, 16
    rng = np.random.default_rng(21)
    src = rng.integers(0, N, size=(N, 2), dtype=np.int64)
    src[-4:, 0] = np.array([N - 1, 0, N - 2, 1])  # the last rows read the first and the last rows
    src[:4, 1] = np.array([N - 1, N - 2, N - 3, N - 4])
    indptr = np.arange(0, 2 * N + 1, 2, dtype=np.int32)
    indices = src.reshape(-1).astype(np.int32)
    g = dfgnn.Graph(indptr, indices)
    L = dfgnn.Layer("gt", H, D, scale=0.25)
    gen = torch.Generator(device="cuda").manual_seed(5)
    q, k, v, d_out = (torch.randn((N, H, D), device="cuda", generator=gen) for _ in range(4))
    out, rmax, rsum = g.forward(L, q, k, v)
    grads = g.backward(L, q, k, v, None, None, out, rmax, rsum, d_out)
    torch.cuda.synchronize()

    rows = np.unique(np.concatenate([np.arange(4), np.arange(N - 4, N), rng.integers(0, N, 24)]))
    cols = np.array([0, 1, N - 2, N - 1, int(src[12345, 0])])
    edge_rows = np.repeat(np.arange(N, dtype=np.int64), 2)
    feed = np.unique(edge_rows[np.isin(indices, cols)])
    need = np.union1d(rows, feed)  # rows whose neighbourhoods the oracle evaluates
    nb = src[need].reshape(-1)
    nodes, inv = np.unique(np.concatenate([need, cols, nb]), return_inverse=True)
    new_rows = inv[:need.size]
    new_nb = inv[need.size + cols.size:]
    sub = from_edge_list(nodes.size, new_nb, np.repeat(new_rows, 2), sort=False)
    pick = torch.from_numpy(nodes).cuda()
    f64 = lambda t: t[pick].cpu().numpy().astype(np.float64)
    import oracle
    OL = oracle.Layer("gt", H, D, scale=0.25)
    kw = dict(x=f64(q), k=f64(k), v=f64(v))
    fw = oracle.forward(OL, sub.indptr, sub.indices, **kw)
    bw = oracle.backward(OL, sub.indptr, sub.indices, d_out=f64(d_out), **kw)
    from gpu_harness import assert_close
    at = lambda ids: np.searchsorted(nodes, ids)
    assert_close("out", f64(out)[at(rows)], fw["out"][at(rows)], "f32")
    assert_close("row_sum", rsum[pick].cpu().numpy()[at(rows)], fw["row_sum"][at(rows)], "f32")
    assert_close("d_x", f64(grads["d_x"])[at(rows)], bw["d_x"][at(rows)], "f32")
    assert_close("d_k", f64(grads["d_k"])[at(cols)], bw["d_k"][at(cols)], "f32")
    assert_close("d_v", f64(grads["d_v"])[at(cols)], bw["d_v"][at(cols)], "f32")
    g.close()


def test_edge_count_just_below_the_int32_limit():
    """2.14 billion edges (99.7 % of the documented maximum of 2^31 - 2^20): every row is a super row, so the
    scheduler, the CSC transpose, the chunk pass and the merge all run at the largest index values.  The
    graph is drawn on the GPU; the oracle evaluates sampled rows and every row that feeds a sampled column."""
    import torch
    import oracle
    from gpu_harness import assert_close
    N, deg, H, D = 1000000, 2140, 1, 4
    E = N * deg
    gen = torch.Generator(device="cuda").manual_seed(9)
    indices = torch.randint(0, N, (E,), dtype=torch.int32, device="cuda", generator=gen)
    indptr = torch.arange(0, E + 1, deg, dtype=torch.int64, device="cuda").to(torch.int32)
    g = dfgnn.Graph(indptr, indices)
    assert g.query("n_super_rows") == N
    L = dfgnn.Layer("gt", H, D, scale=0.5)
    q, k, v, d_out = (torch.randn((N, H, D), device="cuda", generator=gen) for _ in range(4))
    out, rmax, rsum = g.forward(L, q, k, v)
    grads = g.backward(L, q, k, v, None, None, out, rmax, rsum, d_out)
    torch.cuda.synchronize()

    rows = np.array([0, 1, 499999, N - 2, N - 1])
    cols = np.array([int(indices[0]), int(indices[E - 1])])  # sources of the first and of the last edge
    feed = []
    quarter = N // 4 * deg  # positions are searched in four slices to stay far below 2^31 elements per call
    for j in cols:
        for part in range(4):
            pos = (indices[part * quarter:(part + 1) * quarter] == int(j)).nonzero().flatten() + part * quarter
            feed.append(torch.div(pos, deg, rounding_mode="floor").unique().cpu().numpy())
    need = np.unique(np.concatenate([rows] + feed))
    lists = indices.view(N, deg)[torch.from_numpy(need).cuda()].cpu().numpy()  # whole neighbourhoods of those rows
    sub_ptr = np.zeros(N + 1, dtype=np.int64)
    sub_ptr[need + 1] = deg
    sub_ptr = np.cumsum(sub_ptr)
    f64 = lambda t: t.cpu().numpy().astype(np.float64)
    OL = oracle.Layer("gt", H, D, scale=0.5)
    kw = dict(x=f64(q), k=f64(k), v=f64(v))
    fw = oracle.forward(OL, sub_ptr, lists.reshape(-1), **kw)
    bw = oracle.backward(OL, sub_ptr, lists.reshape(-1), d_out=f64(d_out), **kw)
    assert_close("out", f64(out)[rows], fw["out"][rows], "f32")
    assert_close("row_sum", f64(rsum)[rows], fw["row_sum"][rows], "f32")
    assert_close("d_x", f64(grads["d_x"])[rows], bw["d_x"][rows], "f32")
    assert_close("d_k", f64(grads["d_k"])[cols], bw["d_k"][cols], "f32")
    assert_close("d_v", f64(grads["d_v"])[cols], bw["d_v"][cols], "f32")
    g.close()
