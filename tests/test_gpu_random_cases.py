"""Seeded random combinations of model, precision, shape, graph kind, schedule and options, each checked
element by element against the oracle (forward, every gradient, attention weights).  The fixed cases of the
other files cover every feature alone; this file covers their combinations."""
import os

import numpy as np
import pytest

import oracle
import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, make_features
from dfgnn_synth.workloads import Workload
from gpu_harness import run_gpu, run_oracle, compare_all, gpu_layer, oracle_layer, to_device, to_host, assert_close

pytestmark = pytest.mark.gpu

SHAPES = {  # (H, D) the kernels accept: a head is a power-of-two number of 16-byte lanes
    "f32": [(1, 4), (2, 4), (3, 8), (8, 8), (1, 64), (8, 16), (4, 32), (5, 16), (2, 128), (8, 64), (16, 16)],
    "bf16": [(1, 8), (2, 8), (3, 16), (8, 16), (1, 64), (4, 32), (16, 8), (2, 128), (16, 64), (6, 16)],
}
KINDS = ["random", "hub", "dups", "unsorted", "chain", "selfloop"]
SCALES = {"gt": None, "gat": 1.0, "agnn": 1.3, "gatv2": 1.0}


def compare_with_oracle(res, ref, w, graph):
    return compare_all(res, ref, w)


def draw_case(seed):
    rng = np.random.default_rng([2024, seed])
    model = ["gt", "gat", "agnn", "gatv2"][seed % 4]
    dtype = "bf16" if rng.random() < 0.4 else "f32"
    H, D = SHAPES[dtype][int(rng.integers(len(SHAPES[dtype])))]
    if dtype == "bf16" and seed % 3 == 0:  # a third of the 16-bit cases store fp16 (same shapes)
        dtype = "f16"
    kind = KINDS[int(rng.integers(len(KINDS)))]
    n = int(rng.integers(8, 400))
    T = int(rng.choice([4, 8, 16, 64, 0]))          # 0: library default
    C = 0 if T == 0 else int(rng.choice([3, 5, 8, 16]))
    flags = (1 if rng.random() < 0.2 else 0) | (16 if rng.random() < 0.3 else 0)
    bias = bool(rng.random() < 0.35)
    return model, dtype, H, D, kind, n, T, C, flags, bias


@pytest.mark.parametrize("seed", range(int(os.environ.get("DFGNN_RANDOM_CASES", "96"))))  # more seeds on request
def test_random_case(seed):
    import torch
    model, dtype, H, D, kind, n, T, C, flags, bias = draw_case(seed)
    graph = tiny_graph(kind, seed=seed, n=n)
    scale = SCALES[model] if SCALES[model] is not None else float(D) ** -0.5
    w = Workload("random", 500 + seed, model, H, D, dtype, scale)
    feats = make_features(w, graph.n)
    if bias:
        rng = np.random.default_rng([7, seed])
        feats["edge_bias"] = rng.standard_normal((graph.nnz, H)).astype(np.float32)
    case = f"{model} {dtype} H={H} D={D} {kind} n={n} T={T} C={C} flags={flags} bias={bias}"
    print(case, flush=True)
    res, g = run_gpu(graph, w, feats, dfgnn.SchedParams(T, C, flags))
    compare_with_oracle(res, run_oracle(graph, w, feats), w, graph)
    # attention weights from the same call's statistics
    L = gpu_layer(w)
    f32 = lambda name: None if name not in feats else torch.from_numpy(feats[name]).cuda()
    x = to_device(feats["q"] if model == "gt" else feats["feat"], dtype)
    k = to_device(feats["k"], dtype) if model in ("gt", "gatv2") else None
    rmax = torch.from_numpy(res["row_max"].astype(np.float32)).cuda()
    rsum = torch.from_numpy(res["row_sum"].astype(np.float32)).cuda()
    p = to_host(g.attention(L, x, k, f32("a_l"), f32("a_r"), rmax, rsum, edge_bias=f32("edge_bias")))
    kw = dict(x=feats["q"] if model == "gt" else feats["feat"], k=feats.get("k"), v=feats.get("v"),
              a_l=feats.get("a_l"), a_r=feats.get("a_r"), edge_bias=feats.get("edge_bias"))
    kw = {a: (None if b is None else np.asarray(b, dtype=np.float64)) for a, b in kw.items()}
    p_ref = oracle.forward(oracle_layer(w), graph.indptr, graph.indices, want_p=True, **kw)["p"]
    if graph.nnz:
        assert_close("p", p, p_ref, "f32")
    g.close()


def draw_batch(seed):
    rng = np.random.default_rng([2025, seed])
    dtype = "bf16" if rng.random() < 0.5 else "f32"
    H = int(rng.choice([1, 2, 3, 4, 8]))
    D = int(rng.choice([16, 32, 64]))
    if H * D > (256 if dtype == "f32" else 512):  # keep the row within one wavefront for the general kernels too
        H = 1
    n_graphs = int(rng.integers(1, 30))
    hi = int(rng.choice([5, 16, 17, 40, 64, 65, 130, 300]))
    lo = int(rng.integers(1, hi + 1))
    density = float(rng.choice([0.03, 0.1, 0.3, 0.7, 1.0]))
    return dtype, H, D, n_graphs, lo, hi, density


@pytest.mark.parametrize("seed", range(int(os.environ.get("DFGNN_RANDOM_BATCHES", "48"))))
def test_random_batch_on_the_dense_tile_kernels(seed):
    """Batches of small graphs on the MFMA kernels (forced, so that sparse batches take them too): LDS-staged
    bf16 up to 64 nodes, streaming fp32 / bf16 up to 512 nodes."""
    from dfgnn_synth import batched_small_graphs
    dtype, H, D, n_graphs, lo, hi, density = draw_batch(seed)
    graph = batched_small_graphs(n_graphs, lo, hi, density, seed=seed)
    w = Workload("batch", 700 + seed, "gt", H, D, dtype, float(D) ** -0.5)
    feats = make_features(w, graph.n)
    print(f"{dtype} H={H} D={D} graphs={n_graphs} nodes {lo}-{hi} density {density} N={graph.n} E={graph.nnz}", flush=True)
    res, g = run_gpu(graph, w, feats, sched=dfgnn.SchedParams(flags=4))
    assert g.query("n_batch_dense") == 1
    compare_with_oracle(res, run_oracle(graph, w, feats), w, graph)
    g.close()
