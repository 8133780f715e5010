"""Parity of the GATv2 layer (scores sum_d a_d LeakyReLU(x_i,d + k_j,d), the GAT-family variant cited in
Sec. 1) with the CPU oracle, through the C ABI: forward, both feature gradients and the gradient of a."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, complete_graph, make_workload, make_features
from dfgnn_synth.workloads import make_graph, Workload
from gpu_harness import run_gpu, run_oracle, compare_all

pytestmark = pytest.mark.gpu


def v2_workload(H, D, dtype="f32", neg_slope=0.2):
    return Workload("tiny", 93, "gatv2", H, D, dtype, 1.0, neg_slope=neg_slope)


@pytest.mark.parametrize("H,D", [(1, 64), (8, 16), (8, 8), (2, 4), (3, 8), (4, 32), (1, 256)])
@pytest.mark.parametrize("kind", ["random", "hub", "dups", "unsorted", "empty", "selfloop"])
def test_tiny_graphs_f32(H, D, kind):
    graph = tiny_graph(kind, seed=7, n=70)
    w = v2_workload(H, D)
    feats = make_features(w, graph.n)
    # threshold 8 / chunk 5: hub rows and columns go through the chunk + merge path with ragged chunks
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


@pytest.mark.parametrize("H,D", [(8, 16), (1, 8), (3, 16), (2, 64)])
@pytest.mark.parametrize("kind", ["hub", "random"])
def test_tiny_graphs_bf16(H, D, kind):
    graph = tiny_graph(kind, seed=8, n=70)
    w = v2_workload(H, D, "bf16")
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5))
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


def test_complete_graph_and_slopes():
    graph = complete_graph(67)
    for slope in (0.2, 1.0, 0.0):  # 1.0: the score is separable (GAT with a_l = a_r); 0.0: ReLU
        w = v2_workload(2, 16, neg_slope=slope)
        feats = make_features(w, graph.n)
        for sched in (None, dfgnn.SchedParams(32, 16)):
            res, g = run_gpu(graph, w, feats, sched)
            compare_all(res, run_oracle(graph, w, feats), w)
            g.close()


@pytest.mark.parametrize("name,shrink,dtype", [("cfg3", 8, "f32"), ("cfg3", 1, "f32"), ("cfg4", 16, "f32"),
                                               ("cfg1", 1, "f32"), ("cfg3", 8, "bf16")])
def test_workload_graphs(name, shrink, dtype):
    """The benchmark graphs with a GATv2 layer of the same head shape (default scheduling parameters)."""
    base = make_workload(name, shrink=shrink)
    w = make_workload(name, shrink=shrink, model="gatv2", scale=1.0, dtype=dtype)
    graph = make_graph(base)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats)
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


def test_argument_checks():
    import torch
    graph = tiny_graph("random", seed=1, n=20)
    w = v2_workload(2, 16)
    feats = make_features(w, graph.n)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    L = dfgnn.Layer("gatv2", 2, 16)
    x = torch.from_numpy(feats["feat"]).cuda()
    k = torch.from_numpy(feats["k"]).cuda()
    a = torch.from_numpy(feats["a_l"]).cuda()
    with pytest.raises(dfgnn.DfgnnError):
        g.forward(L, x, None, None, a, None)  # source-side features missing
    with pytest.raises(dfgnn.DfgnnError):
        g.forward(L, x, k, None, a, a)  # a second attention vector is not part of the model
    with pytest.raises(dfgnn.DfgnnError):
        g.forward(L, x, k, k, a, None)  # no separate value tensor
    g.close()


def test_autograd_wrapper():
    import torch
    from paper_2411_16127_amd.autograd import gatv2_conv
    graph = tiny_graph("hub", seed=3, n=50)
    w = v2_workload(2, 16)
    feats = make_features(w, graph.n)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    x = torch.from_numpy(feats["feat"]).cuda().requires_grad_()
    k = torch.from_numpy(feats["k"]).cuda().requires_grad_()
    a = torch.from_numpy(feats["a_l"]).cuda().requires_grad_()
    out = gatv2_conv(g, x, k, a, 0.2)
    (out * torch.from_numpy(feats["d_out"]).cuda()).sum().backward()
    ref = run_oracle(graph, w, feats)
    res = {"out": out.detach().cpu().numpy(), "d_x": x.grad.cpu().numpy(), "d_k": k.grad.cpu().numpy(),
           "d_a_l": a.grad.cpu().numpy()}
    compare_all(res, ref, w, keys=list(res))
    g.close()
