"""The autograd wrapper gives the same gradients as the oracle when driven through torch's backward()."""
import numpy as np
import pytest

import oracle
import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph
from gpu_harness import assert_close

pytestmark = pytest.mark.gpu


def test_autograd_wrappers_match_the_oracle():
    import torch
    from paper_2411_16127_amd.autograd import gt_conv, gat_conv, agnn_conv
    graph = tiny_graph("hub", seed=8, n=60)
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(8, 4))
    H, D = 2, 16
    rng = np.random.default_rng(3)
    mk = lambda *s: rng.standard_normal(s).astype(np.float32)
    q, k, v, w, a_l, a_r = mk(graph.n, H, D), mk(graph.n, H, D), mk(graph.n, H, D), mk(graph.n, H, D), mk(H, D), mk(H, D)
    up = lambda a: torch.from_numpy(a).cuda().requires_grad_(True)

    tq, tk, tv = up(q), up(k), up(v)
    out = gt_conv(g, tq, tk, tv)
    (out * torch.from_numpy(w).cuda()).sum().backward()
    L = oracle.Layer("gt", H, D, scale=D ** -0.5)
    ref = oracle.backward(L, graph.indptr, graph.indices, x=q, k=k, v=v, d_out=w)
    for name, t in (("d_x", tq), ("d_k", tk), ("d_v", tv)):
        assert_close(name, t.grad.cpu().numpy(), ref[name], "f32")

    tx, tal, tar = up(q), up(a_l), up(a_r)
    out = gat_conv(g, tx, tal, tar, 0.2)
    (out * torch.from_numpy(w).cuda()).sum().backward()
    ref = oracle.backward(oracle.Layer("gat", H, D), graph.indptr, graph.indices, x=q, a_l=a_l, a_r=a_r, d_out=w)
    for name, t in (("d_x", tx), ("d_a_l", tal), ("d_a_r", tar)):
        assert_close(name, t.grad.cpu().numpy(), ref[name], "f32")

    th, beta = up(q), torch.tensor(1.3, device="cuda", requires_grad=True)
    out = agnn_conv(g, th, beta)
    (out * torch.from_numpy(w).cuda()).sum().backward()
    ref = oracle.backward(oracle.Layer("agnn", H, D, scale=1.3), graph.indptr, graph.indices, x=q, d_out=w)
    assert_close("d_x", th.grad.cpu().numpy(), ref["d_x"], "f32")
    assert_close("d_scale", beta.grad.cpu().numpy().reshape(1), np.array([ref["d_scale"]]), "f32")
    g.close()
