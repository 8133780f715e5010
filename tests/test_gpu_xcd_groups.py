"""XCD-local runs of the work list (graphs whose numbering is local): detection at graph creation, and
bit-identical results with the remapping on and off."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import make_workload, make_features
from dfgnn_synth.workloads import make_graph
from gpu_harness import run_gpu, run_oracle, compare_all

pytestmark = pytest.mark.gpu

NO_XCD_GROUPS = 16


def test_detection():
    batch = make_graph(make_workload("cfg2"))  # block-diagonal: every edge stays within 40 node ids
    g = dfgnn.Graph(batch.indptr, batch.indices)
    assert g.query("n_xcd_group") == 32
    g.close()
    g = dfgnn.Graph(batch.indptr, batch.indices, dfgnn.SchedParams(0, 0, NO_XCD_GROUPS))
    assert g.query("n_xcd_group") == 0
    g.close()
    scattered = make_graph(make_workload("cfg3"))  # 169,343 randomly numbered nodes: 5 % of the edges are near
    g = dfgnn.Graph(scattered.indptr, scattered.indices)
    assert g.query("n_xcd_group") == 0
    g.close()


@pytest.mark.parametrize("name,overrides", [("cfg2", {}), ("cfg2", {"dtype": "f32", "n_min": 60, "n_max": 90, "density": 0.1}),
                                            ("cfg4", {"shrink": 256})])
def test_results_do_not_depend_on_the_mapping(name, overrides):
    """Every row is computed by the same code whichever workgroup picks it up, and partial results are
    combined in a fixed order: outputs are equal bit for bit.  The shrunk cfg4 graph (3,906 nodes, hub rows
    in chunks) has all three kinds of work items in one launch."""
    w = make_workload(name, **overrides)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    on, g1 = run_gpu(graph, w, feats, dfgnn.SchedParams(64, 32, 0), use_batch=False)
    off, g2 = run_gpu(graph, w, feats, dfgnn.SchedParams(64, 32, NO_XCD_GROUPS), use_batch=False)
    assert g1.query("n_xcd_group") == 32 and g2.query("n_xcd_group") == 0
    for key in on:
        assert np.array_equal(on[key], off[key], equal_nan=True), key
    compare_all(on, run_oracle(graph, w, feats), w)
    g1.close(); g2.close()
