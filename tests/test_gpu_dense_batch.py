"""Dense-tile (MFMA) kernels for batches of small graphs: parity with the oracle, agreement with the
general kernels, and the conditions under which the library uses them."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import batched_small_graphs, from_edge_list, make_workload, make_features
from dfgnn_synth.workloads import make_graph, Workload
from gpu_harness import run_gpu, run_oracle, compare_all

pytestmark = pytest.mark.gpu

FORCE = dfgnn.SchedParams(flags=4)  # dense-tile kernels also below the edges-per-graph count from which they pay


def gt_bf16(H, D):
    return Workload("batch", 91, "gt", H, D, "bf16", float(D) ** -0.5)


@pytest.mark.parametrize("H,D", [(8, 16), (1, 16), (3, 16), (4, 32), (1, 32)])
@pytest.mark.parametrize("sizes", [(10, 40), (1, 5), (60, 64), (16, 16), (17, 33)])
def test_dense_batch_matches_oracle(H, D, sizes):
    graph = batched_small_graphs(37, sizes[0], sizes[1], 0.3, seed=5)
    w = gt_bf16(H, D)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, sched=FORCE)
    assert g.query("n_batch_dense") == 1
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


def test_dense_batch_with_empty_rows_and_sparse_graphs():
    # density 0.05 without forcing self-loops: many rows have no edge at all
    rng = np.random.default_rng(4)
    sizes = rng.integers(5, 50, size=20)
    bp = np.concatenate([[0], np.cumsum(sizes)])
    src, dst = [], []
    for b in range(20):
        adj = rng.random((sizes[b], sizes[b])) < 0.05
        d, s = np.nonzero(adj)
        src.append(s + bp[b]); dst.append(d + bp[b])
    graph = from_edge_list(int(bp[-1]), np.concatenate(src), np.concatenate(dst), batch_ptr=bp)
    assert (graph.degrees() == 0).sum() > 20
    w = gt_bf16(2, 16)
    feats = make_features(w, graph.n)
    res, g = run_gpu(graph, w, feats, sched=FORCE)
    assert g.query("n_batch_dense") == 1
    compare_all(res, run_oracle(graph, w, feats), w)
    g.close()


def test_dense_and_general_paths_agree_on_cfg2():
    w = make_workload("cfg2")
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    dense, g1 = run_gpu(graph, w, feats, sched=FORCE)
    general, g2 = run_gpu(graph, w, feats, use_batch=False)
    off, g3 = run_gpu(graph, w, feats, sched=dfgnn.SchedParams(flags=2))
    auto, g4 = run_gpu(graph, w, feats)  # 230 edges per graph: below the count from which the dense kernels pay
    assert g1.query("n_batch_dense") == 1 and g2.query("n_batch_dense") == 0 and g3.query("n_batch_dense") == 1
    ref = run_oracle(graph, w, feats)
    for res in (dense, general, off, auto):
        compare_all(res, ref, w)
    for key in general:
        assert np.array_equal(general[key], off[key]), key   # the ablation flag really selects the general kernels
        assert np.array_equal(general[key], auto[key]), key  # and so does the edges-per-graph rule here
    assert any(not np.array_equal(general[key], dense[key]) for key in general)  # the forced run took the other path
    g1.close(); g2.close(); g3.close(); g4.close()


def test_dense_path_is_chosen_for_dense_enough_batches():
    graph = batched_small_graphs(64, 50, 64, 0.4, seed=6)  # ~1,300 edges per graph
    w = gt_bf16(8, 16)
    feats = make_features(w, graph.n)
    auto, g1 = run_gpu(graph, w, feats)
    off, g2 = run_gpu(graph, w, feats, sched=dfgnn.SchedParams(flags=2))
    ref = run_oracle(graph, w, feats)
    compare_all(auto, ref, w)
    compare_all(off, ref, w)
    assert any(not np.array_equal(auto[key], off[key]) for key in auto)
    g1.close(); g2.close()


def test_layers_outside_the_dense_path_still_use_the_general_kernels():
    graph = batched_small_graphs(30, 10, 40, 0.3, seed=9)
    for w in (Workload("b", 92, "gt", 2, 16, "f32", 0.25), Workload("b", 92, "gat", 2, 16, "bf16", 1.0),
              Workload("b", 92, "gt", 2, 64, "bf16", 0.125)):
        feats = make_features(w, graph.n)
        res, g = run_gpu(graph, w, feats)
        compare_all(res, run_oracle(graph, w, feats), w)
        g.close()


def test_large_graphs_and_repeated_edges_switch_the_dense_path_off():
    big = batched_small_graphs(6, 60, 90, 0.2, seed=2)  # some graphs exceed 64 nodes
    w = gt_bf16(2, 16)
    feats = make_features(w, big.n)
    res, g = run_gpu(big, w, feats)
    assert g.query("n_batch_dense") == 0
    compare_all(res, run_oracle(big, w, feats), w)
    g.close()
    small = batched_small_graphs(6, 10, 20, 0.3, seed=2)
    rows = small.rows_of_edges()
    dup = from_edge_list(small.n, np.concatenate([small.indices, small.indices[:7]]),
                         np.concatenate([rows, rows[:7]]), batch_ptr=small.batch_ptr)
    feats = make_features(w, dup.n)
    res, g = run_gpu(dup, w, feats)
    assert g.query("n_batch_dense") == 0
    compare_all(res, run_oracle(dup, w, feats), w)
    g.close()


def test_set_batch_rejects_bad_input():
    graph = batched_small_graphs(5, 10, 20, 0.3, seed=3)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    import torch
    def status(bp):
        t = torch.tensor(bp, dtype=torch.int32, device="cuda")
        with pytest.raises(dfgnn.DfgnnError) as e:
            dfgnn.graph_set_batch(g.handle, t, len(bp) - 1)
        return e.value.status
    good = graph.batch_ptr.tolist()
    assert status([1] + good[1:]) == 1                      # does not start at 0
    assert status(good[:-1] + [good[-1] - 1]) == 1          # does not end at N
    assert status([0, good[2], good[1]] + good[3:]) == 1    # decreases
    shifted = list(good); shifted[1] += 3                    # boundary cuts through a graph: edges cross
    assert status(shifted) == 1
    keep = torch.tensor(good, dtype=torch.int32, device="cuda")
    dfgnn.graph_set_batch(g.handle, keep, len(good) - 1)     # the well-formed one is accepted afterwards
    assert g.query("n_batch_dense") == 1
    dfgnn.graph_set_batch(g.handle, None, 0)
    assert g.query("n_batch_dense") == 0
    g.close()
