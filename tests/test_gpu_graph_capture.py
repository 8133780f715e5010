"""The layer calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a forward + backward step can be captured into a HIP graph and replayed."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import make_workload, make_features
from dfgnn_synth.workloads import make_graph

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,shrink", [("cfg1", 1), ("cfg3", 16), ("cfg4", 64)])
def test_step_replays_from_a_hip_graph(name, shrink):
    import torch
    w = make_workload(name, shrink=shrink)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(64, 32))
    L = dfgnn.Layer(w.model, w.H, w.D, dtype=w.dtype, scale=w.scale, neg_slope=w.neg_slope, eps=w.eps)
    dev = lambda a: torch.from_numpy(a).cuda()
    x = dev(feats["q"] if w.model == "gt" else feats["feat"])
    k = dev(feats["k"]) if w.model == "gt" else None
    v = dev(feats["v"]) if w.model == "gt" else None
    a_l = dev(feats["a_l"]) if w.model == "gat" else None
    a_r = dev(feats["a_r"]) if w.model == "gat" else None
    d_out = dev(feats["d_out"])
    N, H = graph.n, w.H
    out = torch.empty_like(x); rmax = torch.empty(N, H, device="cuda"); rsum = torch.empty(N, H, device="cuda")
    d_x = torch.empty_like(x)
    d_k = torch.empty_like(x) if w.model == "gt" else None
    d_v = torch.empty_like(x) if w.model == "gt" else None
    d_al = torch.empty(H, w.D, device="cuda") if w.model == "gat" else None
    d_ar = torch.empty(H, w.D, device="cuda") if w.model == "gat" else None
    d_s = torch.empty(1, device="cuda") if w.model == "agnn" else None
    fb, bb = dfgnn.workspace_bytes(g.handle, L)
    ws = torch.empty(max(fb, bb, 256), dtype=torch.uint8, device="cuda")
    results = [t for t in (out, rmax, rsum, d_x, d_k, d_v, d_al, d_ar, d_s) if t is not None]

    def step(stream):
        dfgnn.forward(g.handle, L, x, k, v, a_l, a_r, out, rmax, rsum, ws, ws.numel(), stream)
        dfgnn.backward(g.handle, L, x, k, v, a_l, a_r, out, rmax, rsum, d_out, d_x, d_k, d_v, d_al, d_ar, d_s, ws,
                       ws.numel(), stream)

    step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    eager = [t.clone() for t in results]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    cg = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(side)  # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(cg, stream=side):
            step(side)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in results:
            t.fill_(float("nan"))      # eager work between replays
        torch.cuda.synchronize()
        cg.replay()
        torch.cuda.synchronize()
        for got, want in zip(results, eager):
            assert torch.equal(got, want), (name, rep)  # same kernels, same order: bit-identical
    g.close()


def test_agnn_beta_on_the_device_is_read_at_replay_time():
    """AGNN with beta passed as a device pointer (a_l): the value is read by the kernels, so a captured step
    follows an in-place update of beta between replays; each replay equals an eager call with that beta as the
    layer's host-side scale, bit for bit."""
    import torch
    w = make_workload("cfg4", shrink=64)
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(64, 32))
    x = torch.from_numpy(feats["feat"]).cuda()
    d_out = torch.from_numpy(feats["d_out"]).cuda()
    N, H = graph.n, w.H
    beta = torch.tensor([1.0], device="cuda")

    def buffers():
        return (torch.empty_like(x), torch.empty(N, H, device="cuda"), torch.empty(N, H, device="cuda"),
                torch.empty_like(x), torch.empty(1, device="cuda"))

    def step(L, a_l, bufs, stream):
        out, rmax, rsum, d_x, d_s = bufs
        dfgnn.forward(g.handle, L, x, None, None, a_l, None, out, rmax, rsum, ws, ws.numel(), stream)
        dfgnn.backward(g.handle, L, x, None, None, a_l, None, out, rmax, rsum, d_out, d_x, None, None, None, None, d_s,
                       ws, ws.numel(), stream)

    L_dev = dfgnn.Layer("agnn", w.H, w.D, scale=123.0, eps=w.eps)  # the host-side value must be ignored
    fb, bb = dfgnn.workspace_bytes(g.handle, L_dev)
    ws = torch.empty(max(fb, bb, 256), dtype=torch.uint8, device="cuda")
    captured = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    cg = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(L_dev, beta, captured, side)
        torch.cuda.synchronize()
        with torch.cuda.graph(cg, stream=side):
            step(L_dev, beta, captured, side)
    torch.cuda.synchronize()
    for value in (1.0, 0.5, 2.25):
        beta.fill_(value)
        for t in captured:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        cg.replay()
        torch.cuda.synchronize()
        eager = buffers()
        step(dfgnn.Layer("agnn", w.H, w.D, scale=value, eps=w.eps), None, eager, torch.cuda.current_stream())
        torch.cuda.synchronize()
        for got, want in zip(captured, eager):
            assert torch.equal(got, want), value
    g.close()
