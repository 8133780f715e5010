"""Parity of the attention-weight output (the normalised scores P = Softmax(S) of Eq. 1, per stored edge)
with the oracle: every model, chunked super rows, bf16 tensors, an edge term, rows wider than a wavefront."""
import numpy as np
import pytest

import oracle
import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph, complete_graph, make_workload, make_features
from dfgnn_synth.workloads import make_graph, Workload, round_to_bf16
from gpu_harness import to_device, to_host, gpu_layer, oracle_layer, assert_close

pytestmark = pytest.mark.gpu

SCALES = {"gt": 0.25, "gat": 1.0, "agnn": 1.3, "gatv2": 1.0}


def gpu_attention(graph, w, feats, sched=None):
    import torch
    g = dfgnn.Graph(graph.indptr, graph.indices, sched)
    L = gpu_layer(w)
    f32 = lambda name: None if name not in feats else torch.from_numpy(feats[name]).cuda()
    x = to_device(feats["q"] if w.model == "gt" else feats["feat"], w.dtype)
    k = to_device(feats["k"], w.dtype) if w.model in ("gt", "gatv2") else None
    v = to_device(feats["v"], w.dtype) if w.model == "gt" else None
    a_l, a_r, bias = f32("a_l"), f32("a_r"), f32("edge_bias")
    out, rmax, rsum = g.forward(L, x, k, v, a_l, a_r, edge_bias=bias)
    p = g.attention(L, x, k, a_l, a_r, rmax, rsum, edge_bias=bias)
    torch.cuda.synchronize()
    g.close()
    return to_host(p)


def oracle_attention(graph, w, feats):
    kw = dict(x=feats["q"] if w.model == "gt" else feats["feat"], k=feats.get("k"), v=feats.get("v"),
              a_l=feats.get("a_l"), a_r=feats.get("a_r"), edge_bias=feats.get("edge_bias"))
    kw = {k_: (None if v_ is None else np.asarray(v_, dtype=np.float64)) for k_, v_ in kw.items()}
    return oracle.forward(oracle_layer(w), graph.indptr, graph.indices, want_p=True, **kw)["p"]


def check(graph, w, feats, sched=None):
    got = gpu_attention(graph, w, feats, sched)
    assert got.shape == (graph.nnz, w.H)
    if graph.nnz == 0:
        return
    ref = oracle_attention(graph, w, feats)
    # weights are in [0, 1]: the fp32 bound as stated; bf16 inputs are exact in both paths and the weights
    # are written in fp32, so the same bound holds
    assert_close("p", got, ref, "f32")
    rows = graph.rows_of_edges()
    for h in range(w.H):
        total = np.bincount(rows, weights=got[:, h], minlength=graph.n)
        np.testing.assert_allclose(total[np.diff(graph.indptr) > 0], 1.0, rtol=2e-5)


def add_bias(w, graph, feats, seed=3):
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence([w.seed + 11, seed])))
    feats["edge_bias"] = rng.standard_normal((graph.nnz, w.H), dtype=np.float32)
    return feats


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("H,D", [(1, 64), (8, 16), (3, 8), (2, 4), (4, 128)])
@pytest.mark.parametrize("kind", ["random", "hub", "dups", "unsorted", "empty"])
def test_tiny_graphs_f32(model, H, D, kind):
    graph = tiny_graph(kind, seed=12, n=70)
    w = Workload("tiny", 131, model, H, D, "f32", SCALES[model])
    check(graph, w, make_features(w, graph.n), dfgnn.SchedParams(8, 5))  # hub rows are split into chunks


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
@pytest.mark.parametrize("H,D", [(8, 16), (1, 8), (2, 256)])
@pytest.mark.parametrize("bias", [False, True])
def test_tiny_graphs_bf16(model, H, D, bias):
    graph = tiny_graph("hub", seed=13, n=70)
    w = Workload("tiny", 132, model, H, D, "bf16", SCALES[model])
    feats = make_features(w, graph.n)
    check(graph, w, add_bias(w, graph, feats) if bias else feats, dfgnn.SchedParams(8, 5))


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
def test_edge_term_f32(model):
    graph = tiny_graph("hub", seed=14, n=90)
    w = Workload("tiny", 133, model, 4, 16, "f32", SCALES[model])
    check(graph, w, add_bias(w, graph, make_features(w, graph.n)), dfgnn.SchedParams(16, 8))


def test_complete_graph_default_schedule():
    graph = complete_graph(300)  # rows of 300 edges: whole with the default schedule, chunked with (32, 16)
    w = Workload("tiny", 134, "gt", 2, 16, "f32", 0.25)
    feats = make_features(w, graph.n)
    for sched in (None, dfgnn.SchedParams(32, 16), dfgnn.SchedParams(0, 0, 1)):
        check(graph, w, feats, sched)


@pytest.mark.parametrize("name,shrink", [("cfg1", 1), ("cfg2", 8), ("cfg3", 8), ("cfg4", 16), ("cfg5", 256)])
def test_workloads(name, shrink):
    w = make_workload(name, shrink=shrink)
    graph = make_graph(w)
    check(graph, w, make_features(w, graph.n))


def test_statistics_of_the_dense_tile_kernels():
    """A batch of small graphs whose forward pass ran on the dense-tile (MFMA) kernels: their statistics
    feed the attention output like those of the general kernels."""
    import torch
    w = make_workload("cfg2", shrink=8)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(flags=4), batch_ptr=graph.batch_ptr)
    assert g.query("n_batch_dense") == 1
    L = gpu_layer(w)
    q, k, v = (to_device(feats[n], w.dtype) for n in ("q", "k", "v"))
    out, rmax, rsum = g.forward(L, q, k, v)
    got = to_host(g.attention(L, q, k, None, None, rmax, rsum))
    g.close()
    assert_close("p", got, oracle_attention(graph, w, feats), "f32")


def test_cfg4_full_size_sampled():
    """11.2M edges with the default schedule (the launch configuration the benchmark times): the weights of
    sampled rows, among them hub rows of 200,000 edges cut into hundreds of chunks."""
    w = make_workload("cfg4")
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    got = gpu_attention(graph, w, feats)
    deg = graph.degrees()
    rng = np.random.default_rng(78)
    sample = np.unique(np.concatenate([rng.choice(graph.n, 200, replace=False), np.argsort(deg)[-3:]]))
    ref = oracle.forward(oracle_layer(w), graph.indptr, graph.indices, x=feats["feat"].astype(np.float64),
                         rows=sample, want_p=True)["p"]
    edges = np.concatenate([np.arange(graph.indptr[i], graph.indptr[i + 1]) for i in sample])
    assert np.all(np.isfinite(ref[edges]))
    assert_close("p", got[edges], ref[edges], "f32")


def test_argument_errors():
    import torch
    graph = tiny_graph("random", seed=15, n=30)
    w = Workload("tiny", 135, "gt", 2, 16, "f32", 0.25)
    feats = make_features(w, graph.n)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    L = gpu_layer(w)
    q, k, v = (torch.from_numpy(feats[n]).cuda() for n in ("q", "k", "v"))
    out, rmax, rsum = g.forward(L, q, k, v)
    p = torch.empty((graph.nnz, w.H), dtype=torch.float32, device="cuda")
    with pytest.raises(dfgnn.DfgnnError):  # GT needs k
        dfgnn.attention_weights(g.handle, L, q, None, None, None, None, rmax, rsum, p)
    with pytest.raises(dfgnn.DfgnnError):  # no statistics
        dfgnn.attention_weights(g.handle, L, q, k, None, None, None, None, rsum, p)
    with pytest.raises(dfgnn.DfgnnError):  # attention vectors belong to GAT
        dfgnn.attention_weights(g.handle, L, q, k, rsum, None, None, rmax, rsum, p)
    g.close()


@pytest.mark.gpu
@pytest.mark.parametrize("row_bytes", [16, 128, 512, 1024])
def test_gather_yardstick_reads_every_requested_row(row_bytes):
    """dfgnn_probe_gather: the XOR of what all threads read equals the XOR of the requested rows, piece by piece
    (an index of -1 or beyond the table reads nothing); wrong sizes are refused."""
    import torch
    rng = np.random.default_rng(row_bytes)
    n_rows, n_idx = 1000, 12345
    table = rng.integers(0, 2**31 - 1, size=(n_rows, row_bytes // 4), dtype=np.int32)
    idx = rng.integers(0, n_rows, size=n_idx, dtype=np.int32)
    idx[::97] = -1
    idx[5::89] = n_rows + 3
    out = torch.empty(6 * 1024, dtype=torch.int32, device="cuda")  # 6 workgroups
    dfgnn.probe_gather(torch.from_numpy(table).cuda(), row_bytes, torch.from_numpy(idx).cuda(), out)
    got = out.cpu().numpy().reshape(-1, 64, 4)  # wavefront, lane, word
    lpe = row_bytes // 16
    valid = idx[(idx >= 0) & (idx < n_rows)]
    want = np.bitwise_xor.reduce(table[valid], axis=0).reshape(lpe, 4)
    per_piece = np.zeros((lpe, 4), dtype=np.int32)
    for lane in range(64):
        per_piece[lane % lpe] ^= np.bitwise_xor.reduce(got[:, lane, :], axis=0)
    assert np.array_equal(per_piece, want)
    with pytest.raises(dfgnn.DfgnnError):
        dfgnn.probe_gather(torch.from_numpy(table).cuda(), 48, torch.from_numpy(idx).cuda(), out)
    with pytest.raises(dfgnn.DfgnnError):
        dfgnn.probe_gather(torch.from_numpy(table).cuda(), row_bytes, torch.from_numpy(idx).cuda(), out[:16])
