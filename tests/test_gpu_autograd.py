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


@pytest.mark.parametrize("D,dtype", [(7, "f32"), (10, "f32"), (5, "bf16")])
def test_odd_head_widths_are_padded_by_the_wrappers(D, dtype):
    """Head widths that are not a power-of-two number of 16-byte lanes (a classifier layer with 7 outputs):
    the wrappers zero-pad, which changes no score, and cut the result back."""
    import torch
    from paper_2411_16127_amd.autograd import gt_conv, gat_conv, agnn_conv, gatv2_conv
    from dfgnn_synth.workloads import round_to_bf16
    graph = tiny_graph("hub", seed=9, n=50)
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(8, 4))
    H = 2
    rng = np.random.default_rng(4)
    mk = lambda *s: rng.standard_normal(s).astype(np.float32)
    rnd = (lambda a: round_to_bf16(a)) if dtype == "bf16" else (lambda a: a)
    q, k, v, w = (rnd(mk(graph.n, H, D)) for _ in range(4))
    a_l, a_r = mk(H, D), mk(H, D)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    up = lambda a: torch.from_numpy(a).cuda().to(tdt).requires_grad_(True)
    upf = lambda a: torch.from_numpy(a).cuda().requires_grad_(True)
    tw = torch.from_numpy(w).cuda().to(tdt)
    grad = lambda t: t.grad.float().cpu().numpy()

    tq, tk, tv = up(q), up(k), up(v)
    out = gt_conv(g, tq, tk, tv)
    assert out.shape == (graph.n, H, D)
    (out * tw).sum().backward()
    ref = oracle.backward(oracle.Layer("gt", H, D, scale=D ** -0.5), graph.indptr, graph.indices, x=q, k=k, v=v, d_out=w)
    fwd = oracle.forward(oracle.Layer("gt", H, D, scale=D ** -0.5), graph.indptr, graph.indices, x=q, k=k, v=v)
    assert_close("out", out.detach().float().cpu().numpy(), fwd["out"], dtype)
    for name, t in (("d_x", tq), ("d_k", tk), ("d_v", tv)):
        assert_close(name, grad(t), ref[name], dtype)

    tx, tal, tar = up(q), upf(a_l), upf(a_r)
    (gat_conv(g, tx, tal, tar, 0.2) * tw).sum().backward()
    ref = oracle.backward(oracle.Layer("gat", H, D), graph.indptr, graph.indices, x=q, a_l=a_l, a_r=a_r, d_out=w)
    for name, t in (("d_x", tx), ("d_a_l", tal), ("d_a_r", tar)):
        assert_close(name, grad(t), ref[name], dtype)

    tx, tk2, ta = up(q), up(k), upf(a_l)
    (gatv2_conv(g, tx, tk2, ta, 0.2) * tw).sum().backward()
    ref = oracle.backward(oracle.Layer("gatv2", H, D), graph.indptr, graph.indices, x=q, k=k, a_l=a_l, d_out=w)
    for name, t in (("d_x", tx), ("d_k", tk2), ("d_a_l", ta)):
        assert_close(name, grad(t), ref[name], dtype)

    th, beta = up(q), torch.tensor(1.3, device="cuda", requires_grad=True)
    (agnn_conv(g, th, beta) * tw).sum().backward()
    ref = oracle.backward(oracle.Layer("agnn", H, D, scale=1.3), graph.indptr, graph.indices, x=q, d_out=w)
    assert_close("d_x", grad(th), ref["d_x"], dtype)
    assert_close("d_scale", beta.grad.cpu().numpy().reshape(1), np.array([ref["d_scale"]]), dtype)
    g.close()
