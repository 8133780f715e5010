"""The two-kernel forward comparator (edge-parallel SDDMM that writes the scores, then softmax + SpMM;
Sec. 3, parallelism maximization fusion) gives the oracle's forward results like the fused pass does."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, complete_graph, make_workload, make_features
from dfgnn_synth.workloads import make_graph, Workload
from gpu_harness import run_gpu, run_oracle, compare_all

pytestmark = pytest.mark.gpu

SCORES_IN_MEMORY = 8
FORWARD_KEYS = ("out", "row_max", "row_sum")


def small_gt(H, D, dtype="f32"):
    return Workload("tiny", 91, "gt", H, D, dtype, float(1.0 / np.sqrt(D)))


@pytest.mark.parametrize("H,D,dtype", [(1, 64, "f32"), (8, 16, "f32"), (3, 8, "f32"), (2, 128, "f32"),
                                       (8, 16, "bf16"), (1, 8, "bf16")])
@pytest.mark.parametrize("kind", ["random", "hub", "dups", "empty"])
def test_tiny_graphs(H, D, dtype, kind):
    graph = tiny_graph(kind, seed=5, n=70)
    w = small_gt(H, D, dtype)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5, SCORES_IN_MEMORY))
    compare_all(res, run_oracle(graph, w, feats), w)  # backward is the ordinary fused one
    g.close()


def test_complete_graph_and_no_edges():
    w = small_gt(2, 16)
    for graph in (complete_graph(67), tiny_graph("empty", seed=1, n=5)):
        feats = make_features(w, graph.n)
        res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(0, 0, SCORES_IN_MEMORY))
        compare_all(res, run_oracle(graph, w, feats), w, keys=FORWARD_KEYS)
        g.close()


@pytest.mark.parametrize("name,shrink", [("cfg1", 1), ("cfg5", 256), ("cfg2", 8)])
def test_workloads(name, shrink):
    w = make_workload(name, shrink=shrink)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(0, 0, SCORES_IN_MEMORY), use_batch=False)
    compare_all(res, run_oracle(graph, w, feats), w, keys=FORWARD_KEYS)
    g.close()


def test_other_models_ignore_the_switch():
    graph = tiny_graph("hub", seed=6, n=70)
    for model, scale in (("gat", 1.0), ("agnn", 1.3)):
        w = Workload("tiny", 92, model, 2, 16, "f32", scale)
        feats = make_features(w, graph.n)
        res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(8, 5, SCORES_IN_MEMORY))
        compare_all(res, run_oracle(graph, w, feats), w)
        g.close()
