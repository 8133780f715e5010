"""Forward-only graphs (inference): no CSC and no column schedule are built; forward results, statistics and
attention weights are those of an ordinary graph, backward calls are refused."""
import numpy as np
import pytest

import oracle
import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, make_workload, make_features
from dfgnn_synth.workloads import make_graph, Workload
from gpu_harness import to_device, to_host, gpu_layer, oracle_layer, assert_close

pytestmark = pytest.mark.gpu

FORWARD_ONLY = 32
SCALES = {"gt": 0.25, "gat": 1.0, "agnn": 1.3, "gatv2": 1.0}


def forward_on(graph, w, feats, sched, batch_ptr=None):
    import torch
    g = dfgnn.Graph(graph.indptr, graph.indices, sched, batch_ptr=batch_ptr)
    L = gpu_layer(w)
    f32 = lambda name: None if name not in feats else torch.from_numpy(feats[name]).cuda()
    x = to_device(feats["q"] if w.model == "gt" else feats["feat"], w.dtype)
    k = to_device(feats["k"], w.dtype) if w.model in ("gt", "gatv2") else None
    v = to_device(feats["v"], w.dtype) if w.model == "gt" else None
    out, rmax, rsum = g.forward(L, x, k, v, f32("a_l"), f32("a_r"))
    p = g.attention(L, x, k, f32("a_l"), f32("a_r"), rmax, rsum)
    res = {"out": to_host(out), "row_max": to_host(rmax), "row_sum": to_host(rsum), "p": to_host(p)}
    return g, L, (x, k, v, f32("a_l"), f32("a_r"), out, rmax, rsum), res


def oracle_forward(graph, w, feats):
    kw = dict(x=feats["q"] if w.model == "gt" else feats["feat"], k=feats.get("k"), v=feats.get("v"),
              a_l=feats.get("a_l"), a_r=feats.get("a_r"))
    kw = {a: (None if b is None else np.asarray(b, dtype=np.float64)) for a, b in kw.items()}
    return oracle.forward(oracle_layer(w), graph.indptr, graph.indices, want_p=True, **kw)


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_matches_the_oracle_and_backward_is_refused(model, dtype):
    import torch
    graph = tiny_graph("hub", seed=21, n=150)
    w = Workload("tiny", 140, model, 4, 16, dtype, SCALES[model])
    feats = make_features(w, graph.n)
    g, L, t, res = forward_on(graph, w, feats, dfgnn.SchedParams(16, 8, FORWARD_ONLY))  # hub row in chunks
    ref = oracle_forward(graph, w, feats)
    for key in ("out", "row_max", "row_sum"):
        assert_close(key, res[key], ref[key], dtype)
    assert_close("p", res["p"], ref["p"], "f32")
    for what in ("t_indptr", "t_indices", "t_eid", "col_order", "col_chunks"):
        assert g.query(what).numel() == 0
    assert g.query("n_super_cols") == 0 and g.query("n_super_rows") > 0
    x, k, v, a_l, a_r, out, rmax, rsum = t
    with pytest.raises(dfgnn.DfgnnError, match="forward-only"):
        g.backward(L, x, k, v, a_l, a_r, out, rmax, rsum, torch.ones_like(out))
    g.close()


def test_results_equal_those_of_an_ordinary_graph_and_metadata_shrinks():
    w = make_workload("cfg3", shrink=8)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    g1, _, _, plain = forward_on(graph, w, feats, None)
    g2, _, _, fwd_only = forward_on(graph, w, feats, dfgnn.SchedParams(flags=FORWARD_ONLY))
    for key in plain:
        assert np.array_equal(plain[key], fwd_only[key], equal_nan=True), key
    assert np.array_equal(g1.query("row_order").cpu().numpy(), g2.query("row_order").cpu().numpy())
    full, _ = dfgnn.graph_meta_bytes(graph.n, graph.nnz, None)
    small, _ = dfgnn.graph_meta_bytes(graph.n, graph.nnz, dfgnn.SchedParams(flags=FORWARD_ONLY))
    assert small < full - 8 * graph.nnz
    g1.close(); g2.close()


def test_batch_of_small_graphs_on_the_dense_tile_kernels():
    w = make_workload("cfg2", shrink=8)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    g, _, _, res = forward_on(graph, w, feats, dfgnn.SchedParams(flags=FORWARD_ONLY | 4), batch_ptr=graph.batch_ptr)
    assert g.query("n_batch_dense") == 1
    ref = oracle_forward(graph, w, feats)
    for key in ("out", "row_max", "row_sum"):
        assert_close(key, res[key], ref[key], w.dtype)
    g.close()
