"""Parity with the oracle when an additive per-edge term enters the score (edge features in the attention
score, Sec. 1): forward, every gradient of the layer, and the gradient of the term itself (= dS)."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, complete_graph, make_workload, make_features
from dfgnn_synth.workloads import make_graph, Workload, round_to_bf16
from gpu_harness import run_gpu, run_oracle, compare_all

pytestmark = pytest.mark.gpu

SCALES = {"gt": 0.25, "gat": 1.0, "agnn": 1.3, "gatv2": 1.0}


def with_bias(w, graph, seed=5, std=1.0):
    feats = make_features(w, graph.n)
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence([w.seed + 3, seed])))
    feats["edge_bias"] = (rng.standard_normal((graph.nnz, w.H), dtype=np.float32) * np.float32(std))
    return feats


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("H,D", [(1, 64), (8, 16), (3, 8), (2, 4)])
@pytest.mark.parametrize("kind", ["random", "hub", "dups", "unsorted", "empty"])
def test_tiny_graphs_f32(model, H, D, kind):
    graph = tiny_graph(kind, seed=9, n=70)
    w = Workload("tiny", 94, model, H, D, "f32", SCALES[model])
    feats = with_bias(w, graph)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))  # hub rows and columns are split into chunks
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("H,D", [(8, 16), (1, 8)])
def test_tiny_graphs_bf16(model, H, D):
    graph = tiny_graph("hub", seed=10, n=70)
    w = Workload("tiny", 95, model, H, D, "bf16", SCALES[model])
    feats = with_bias(w, graph)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


def test_complete_graph_default_schedule():
    graph = complete_graph(67)
    w = Workload("tiny", 96, "gt", 2, 16, "f32", 0.25)
    feats = with_bias(w, graph)
    for sched in (None, dfgnn.SchedParams(32, 16), dfgnn.SchedParams(0, 0, 1), dfgnn.SchedParams(0, 0, 8)):
        res, g = run_gpu(graph, w, feats, sched)
        compare_all(res, run_oracle(graph, w, feats), w)
        g.close()


@pytest.mark.parametrize("name,shrink", [("cfg1", 1), ("cfg2", 8), ("cfg3", 8), ("cfg4", 16), ("cfg5", 256)])
def test_workloads(name, shrink):
    """The benchmark workloads (reduced) with an edge term; cfg2's batch falls back to the general kernels."""
    w = make_workload(name, shrink=shrink)
    graph = make_graph(w)
    feats = with_bias(w, graph)
    res, g = run_gpu(graph, w, feats)
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


def test_row_constant_bias_changes_nothing():
    """Softmax is invariant to a shift of a whole row: a bias that only depends on the destination leaves
    the output where it was (the two runs differ by rounding only)."""
    w = make_workload("cfg1")
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    base, g = run_gpu(graph, w, feats)
    per_row = np.random.default_rng(3).standard_normal((graph.n, w.H)).astype(np.float32)
    feats["edge_bias"] = np.ascontiguousarray(per_row[graph.rows_of_edges()])
    shifted, _ = run_gpu(graph, w, feats, g=g)
    np.testing.assert_allclose(shifted["out"], base["out"], rtol=2e-5, atol=2e-6)
    np.testing.assert_allclose(shifted["d_edge_bias"].reshape(graph.nnz, w.H).sum(0), 0.0, atol=1e-3)
    g.close()


def test_untrained_term_and_argument_checks():
    import torch
    graph = tiny_graph("random", seed=1, n=30)
    w = Workload("tiny", 97, "gt", 2, 16, "f32", 0.25)
    feats = with_bias(w, graph)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    L = dfgnn.Layer("gt", 2, 16, scale=0.25)
    q, k, v, d_out = (torch.from_numpy(feats[n]).cuda() for n in ("q", "k", "v", "d_out"))
    b = torch.from_numpy(feats["edge_bias"]).cuda()
    out, rmax, rsum = g.forward(L, q, k, v, edge_bias=b)
    res = g.backward(L, q, k, v, None, None, out, rmax, rsum, d_out, edge_bias=b, want_d_edge_bias=False)
    assert "d_edge_bias" not in res
    ref = run_oracle(graph, w, feats)
    np.testing.assert_allclose(res["d_x"].cpu().numpy().astype(np.float64), ref["d_x"], rtol=1e-4, atol=1e-5)
    with pytest.raises(ValueError):
        g.forward(L, q, k, v, edge_bias=b[:-1])  # wrong number of edges
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(dfgnn.DfgnnError):  # a gradient buffer without the term itself
        dfgnn.backward_edge_bias(g.handle, L, q, k, v, None, None, None, out, rmax, rsum, d_out, torch.empty_like(q),
                                 torch.empty_like(q), torch.empty_like(q), None, None, None, torch.empty_like(b), ws,
                                 ws.numel())
    g.close()


def test_autograd_wrapper():
    import torch
    from paper_2411_16127_amd.autograd import gt_conv
    graph = tiny_graph("hub", seed=3, n=50)
    w = Workload("tiny", 98, "gt", 2, 16, "f32", 0.25)
    feats = with_bias(w, graph)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    q, k, v, b = (torch.from_numpy(feats[n]).cuda().requires_grad_() for n in ("q", "k", "v", "edge_bias"))
    out = gt_conv(g, q, k, v, scale=0.25, edge_bias=b)
    (out * torch.from_numpy(feats["d_out"]).cuda()).sum().backward()
    ref = run_oracle(graph, w, feats)
    res = {"out": out.detach().cpu().numpy(), "d_x": q.grad.cpu().numpy(), "d_k": k.grad.cpu().numpy(),
           "d_v": v.grad.cpu().numpy(), "d_edge_bias": b.grad.cpu().numpy()}
    compare_all(res, ref, w, keys=list(res))
    g.close()
