"""The nn modules produce what the oracle gives on their own projected inputs, and train."""
import numpy as np
import pytest

import oracle
import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph
from gpu_harness import assert_close

pytestmark = pytest.mark.gpu


def test_modules_match_the_oracle_on_their_projections():
    import torch
    from paper_2411_16127_amd.nn import GTConv, GATConv, GATv2Conv, AGNNConv
    torch.manual_seed(0)
    graph = tiny_graph("hub", seed=4, n=80)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    feat = torch.randn(graph.n, 24, device="cuda")
    f64 = lambda t: t.detach().cpu().numpy().astype(np.float64)
    H, D = 4, 8

    m = GTConv(24, D, H).cuda()
    out = m(g, feat)
    # the projections recomputed in float64 from the module's parameters (one weight of shape [3, in, H*D])
    q, k, v = ((f64(feat) @ f64(m.w_qkv[i]) + f64(m.b_qkv[i])).reshape(-1, H, D) for i in range(3))
    ref = oracle.forward(oracle.Layer("gt", H, D, scale=D ** -0.5), graph.indptr, graph.indices, x=q, k=k, v=v)
    assert_close("out", f64(out), ref["out"], "f32", tol=(1e-4, 2e-5, 0.0))  # the fp32 projection GEMM rounds the inputs

    m = GATConv(24, 7, 2).cuda()  # 7 features per head: padded inside the wrapper
    out = m(g, feat)
    wh = f64(m.fc(feat)).reshape(-1, 2, 7)
    ref = oracle.forward(oracle.Layer("gat", 2, 7), graph.indptr, graph.indices, x=wh, a_l=f64(m.attn_l), a_r=f64(m.attn_r))
    assert out.shape == (graph.n, 2, 7)
    assert_close("out", f64(out), ref["out"], "f32")

    m = GATv2Conv(24, D, H).cuda()
    out = m(g, feat)
    xd, xs = (f64(lin(feat)).reshape(-1, H, D) for lin in (m.fc_dst, m.fc_src))
    ref = oracle.forward(oracle.Layer("gatv2", H, D), graph.indptr, graph.indices, x=xd, k=xs, a_l=f64(m.attn))
    assert_close("out", f64(out), ref["out"], "f32")

    m = AGNNConv(init_beta=1.5).cuda()
    out = m(g, feat[:, :16])
    ref = oracle.forward(oracle.Layer("agnn", 1, 16, scale=1.5), graph.indptr, graph.indices, x=f64(feat[:, :16]).reshape(-1, 1, 16))
    assert_close("out", f64(out).reshape(-1, 1, 16), ref["out"], "f32")
    g.close()


def test_a_two_layer_model_trains():
    """A few optimiser steps of GAT -> GT on a fixed random regression target lower the loss."""
    import torch
    from paper_2411_16127_amd.nn import GTConv, GATConv
    torch.manual_seed(1)
    graph = tiny_graph("random", seed=5, n=120)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    feat = torch.randn(graph.n, 16, device="cuda")
    target = torch.randn(graph.n, 8, device="cuda")

    class Net(torch.nn.Module):
        def __init__(self):
            super().__init__()
            self.l1 = GATConv(16, 8, 4)
            self.l2 = GTConv(32, 8, 1)

        def forward(self, x):
            h = torch.relu(self.l1(g, x).flatten(1))
            return self.l2(g, h).flatten(1)

    net = Net().cuda()
    opt = torch.optim.Adam(net.parameters(), lr=1e-2)
    losses = []
    for _ in range(30):
        opt.zero_grad()
        loss = ((net(feat) - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert all(np.isfinite(losses)) and losses[-1] < 0.8 * losses[0], losses
    g.close()
