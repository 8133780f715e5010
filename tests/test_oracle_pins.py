"""Pins for the CPU oracle (no GPU): a dense library route, finite differences, invariants, closed forms.

Each test names the passage whose reading it fixes: Eq. 1 (Sec. 2.1) for the layer, Appendix A for
the edge softmax, Appendix B for the backward pass, Sec. 5.1 for the three models' scores; GATv2 is the
second member of the GAT family cited in Sec. 1.
"""
import numpy as np
import pytest

import oracle
from dfgnn_synth import complete_graph, tiny_graph, from_edge_list
from dense_reference import dense_layer

MODELS = ["gt", "gat", "agnn", "gatv2"]


def make_inputs(model, n, H, D, seed):
    rng = np.random.default_rng(seed)
    t = {"x": rng.standard_normal((n, H, D))}
    if model == "gt":
        t["k"] = rng.standard_normal((n, H, D))
        t["v"] = rng.standard_normal((n, H, D))
    if model == "gat":
        t["a_l"] = rng.standard_normal((H, D)) * 0.5
        t["a_r"] = rng.standard_normal((H, D)) * 0.5
    if model == "gatv2":
        t["k"] = rng.standard_normal((n, H, D))
        t["a_l"] = rng.standard_normal((H, D)) * 0.5
    g = rng.standard_normal((n, H, D))
    return t, g


def layer_for(model, H, D):
    scale = {"gt": 1.0 / np.sqrt(D), "gat": 1.0, "agnn": 1.7, "gatv2": 1.0}[model]
    return oracle.Layer(model, H, D, scale=scale, neg_slope=0.2, eps=1e-12)


def run_oracle(layer, g, t, d_out, **kw):
    fw = oracle.forward(layer, g.indptr, g.indices, x=t["x"], k=t.get("k"), v=t.get("v"),
                        a_l=t.get("a_l"), a_r=t.get("a_r"), edge_bias=t.get("edge_bias"), want_p=True)
    bw = oracle.backward(layer, g.indptr, g.indices, x=t["x"], k=t.get("k"), v=t.get("v"),
                         a_l=t.get("a_l"), a_r=t.get("a_r"), edge_bias=t.get("edge_bias"), d_out=d_out,
                         want_ds=True, **kw)
    return fw, bw


# ---------------------------------------------------------------- dense library route (fwd + bwd)
@pytest.mark.parametrize("model", MODELS)
@pytest.mark.parametrize("graph", ["complete", "random", "hub", "chain", "selfloop"])
def test_matches_dense_masked_attention(model, graph):
    H, D = 2, 4
    g = complete_graph(9) if graph == "complete" else tiny_graph(graph, seed=3, n=17)
    t, d_out = make_inputs(model, g.n, H, D, seed=11)
    layer = layer_for(model, H, D)
    fw, bw = run_oracle(layer, g, t, d_out)
    ref, grads = dense_layer(model, g.indptr, g.indices, H, D, layer.scale, layer.neg_slope, layer.eps, t, d_out)
    np.testing.assert_allclose(fw["out"], ref["out"], rtol=1e-11, atol=1e-12)
    has = np.diff(g.indptr) > 0
    np.testing.assert_allclose(fw["row_max"][has], ref["row_max"][has], rtol=1e-12, atol=1e-12)
    assert np.all(np.isneginf(fw["row_max"][~has])) and np.all(fw["row_sum"][~has] == 0)
    np.testing.assert_allclose(bw["d_x"], grads["x"], rtol=1e-9, atol=1e-11)
    if model == "gt":
        np.testing.assert_allclose(bw["d_k"], grads["k"], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(bw["d_v"], grads["v"], rtol=1e-9, atol=1e-11)
    if model == "gat":
        np.testing.assert_allclose(bw["d_a_l"], grads["a_l"], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(bw["d_a_r"], grads["a_r"], rtol=1e-9, atol=1e-11)
    if model == "agnn":
        np.testing.assert_allclose(bw["d_scale"], grads["beta"], rtol=1e-9, atol=1e-11)
    if model == "gatv2":
        np.testing.assert_allclose(bw["d_k"], grads["k"], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(bw["d_a_l"], grads["a_l"], rtol=1e-9, atol=1e-11)


def test_complete_graph_is_dense_softmax_attention():
    """Eq. 1 with A = all ones: O = softmax(scale Q K^T) V, written with plain numpy."""
    n, H, D = 12, 3, 5
    g = complete_graph(n)
    t, d_out = make_inputs("gt", n, H, D, seed=5)
    layer = layer_for("gt", H, D)
    fw, _ = run_oracle(layer, g, t, d_out)
    for h in range(H):
        s = layer.scale * t["x"][:, h] @ t["k"][:, h].T
        p = np.exp(s - s.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        np.testing.assert_allclose(fw["out"][:, h], p @ t["v"][:, h], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(fw["row_max"][:, h], s.max(1), rtol=1e-13)
        np.testing.assert_allclose(fw["row_sum"][:, h], np.exp(s - s.max(1, keepdims=True)).sum(1), rtol=1e-13)


# ---------------------------------------------------------------- finite differences (Appendix B)
def _loss(layer, g, t, d_out):
    fw = oracle.forward(layer, g.indptr, g.indices, x=t["x"], k=t.get("k"), v=t.get("v"),
                        a_l=t.get("a_l"), a_r=t.get("a_r"), edge_bias=t.get("edge_bias"))
    return float((fw["out"] * d_out).sum())


@pytest.mark.parametrize("model", MODELS)
@pytest.mark.parametrize("graph", ["random", "hub", "dups", "unsorted"])
def test_backward_by_central_differences(model, graph):
    H, D = 2, 3
    g = tiny_graph(graph, seed=2, n=14)
    t, d_out = make_inputs(model, g.n, H, D, seed=23)
    layer = layer_for(model, H, D)
    _, bw = run_oracle(layer, g, t, d_out)
    names = {"x": "d_x", "k": "d_k", "v": "d_v", "a_l": "d_a_l", "a_r": "d_a_r", "edge_bias": "ds"}
    step = 1e-6
    rng = np.random.default_rng(0)
    for key in t:
        flat = t[key].reshape(-1)
        picks = rng.choice(flat.size, size=min(flat.size, 40), replace=False)
        for idx in picks:
            keep = flat[idx]
            flat[idx] = keep + step
            up = _loss(layer, g, t, d_out)
            flat[idx] = keep - step
            dn = _loss(layer, g, t, d_out)
            flat[idx] = keep
            fd = (up - dn) / (2 * step)
            an = bw[names[key]].reshape(-1)[idx]
            assert abs(fd - an) <= 2e-7 + 2e-6 * abs(an), (model, graph, key, idx, fd, an)
    if model == "agnn":
        up = _loss(oracle.Layer("agnn", H, D, scale=layer.scale + step), g, t, d_out)
        dn = _loss(oracle.Layer("agnn", H, D, scale=layer.scale - step), g, t, d_out)
        assert abs((up - dn) / (2 * step) - bw["d_scale"]) <= 2e-7 + 2e-6 * abs(bw["d_scale"])


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("model", MODELS)
def test_rows_of_p_sum_to_one_and_ds_rows_sum_to_zero(model):
    H, D = 2, 4
    g = tiny_graph("dups", seed=4, n=20)
    t, d_out = make_inputs(model, g.n, H, D, seed=1)
    fw, bw = run_oracle(layer_for(model, H, D), g, t, d_out)
    rows = g.rows_of_edges()
    for h in range(H):
        psum = np.bincount(rows, weights=fw["p"][:, h], minlength=g.n)
        dssum = np.bincount(rows, weights=bw["ds"][:, h], minlength=g.n)
        has = g.degrees() > 0
        np.testing.assert_allclose(psum[has], 1.0, rtol=1e-13)
        np.testing.assert_allclose(dssum, 0.0, atol=1e-13)


@pytest.mark.parametrize("model", MODELS)
def test_constant_value_column_is_reproduced(model):
    """sum_j p_ij = 1  <=>  a constant column of the aggregated values comes out unchanged (GT only has a
    separate V; for GAT/AGNN the value is the feature itself, so the check is on P above)."""
    if model != "gt":
        pytest.skip("value tensor is not independent of the score for this model")
    H, D = 2, 4
    g = tiny_graph("random", seed=9, n=20)
    t, d_out = make_inputs(model, g.n, H, D, seed=1)
    t["v"][:, :, 1] = 3.25
    fw, _ = run_oracle(layer_for(model, H, D), g, t, d_out)
    has = g.degrees() > 0
    np.testing.assert_allclose(fw["out"][has][:, :, 1], 3.25, rtol=1e-13)
    assert np.all(fw["out"][~has] == 0)


@pytest.mark.parametrize("model", MODELS)
def test_node_relabelling_equivariance(model):
    H, D = 2, 4
    g = tiny_graph("hub", seed=6, n=18)
    t, d_out = make_inputs(model, g.n, H, D, seed=8)
    layer = layer_for(model, H, D)
    fw, bw = run_oracle(layer, g, t, d_out)
    perm = np.random.default_rng(3).permutation(g.n)  # new id of old node v is perm[v]
    rows = g.rows_of_edges()
    g2 = from_edge_list(g.n, perm[g.indices], perm[rows])
    t2 = {}
    for key, val in t.items():
        if key in ("a_l", "a_r"):
            t2[key] = val
        else:
            t2[key] = np.empty_like(val)
            t2[key][perm] = val
    d2 = np.empty_like(d_out)
    d2[perm] = d_out
    fw2, bw2 = run_oracle(layer, g2, t2, d2)
    np.testing.assert_allclose(fw2["out"][perm], fw["out"], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(fw2["row_sum"][perm], fw["row_sum"], rtol=1e-11)
    np.testing.assert_allclose(bw2["d_x"][perm], bw["d_x"], rtol=1e-9, atol=1e-12)
    if model == "gt":
        np.testing.assert_allclose(bw2["d_k"][perm], bw["d_k"], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(bw2["d_v"][perm], bw["d_v"], rtol=1e-9, atol=1e-12)
    if model == "gatv2":
        np.testing.assert_allclose(bw2["d_k"][perm], bw["d_k"], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(bw2["d_a_l"], bw["d_a_l"], rtol=1e-9, atol=1e-12)


def test_score_shift_invariance_gt():
    """Adding one vector c to every K row shifts all scores of row i by scale*q_i.c: P, O unchanged."""
    H, D = 2, 4
    g = tiny_graph("random", seed=1, n=16)
    t, d_out = make_inputs("gt", g.n, H, D, seed=2)
    layer = layer_for("gt", H, D)
    fw, _ = run_oracle(layer, g, t, d_out)
    t2 = dict(t)
    t2["k"] = t["k"] + np.array([0.3, -1.1, 2.0, 0.7])
    fw2, _ = run_oracle(layer, g, t2, d_out)
    np.testing.assert_allclose(fw2["out"], fw["out"], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(fw2["p"], fw["p"], rtol=1e-11)


def test_large_scores_stay_finite():
    H, D = 1, 4
    g = tiny_graph("hub", seed=1, n=16)
    t, d_out = make_inputs("gt", g.n, H, D, seed=2)
    t["x"] *= 1e3
    fw, bw = run_oracle(oracle.Layer("gt", H, D, scale=1.0), g, t, d_out)
    has = g.degrees() > 0
    assert np.all(np.isfinite(fw["out"])) and np.all(np.isfinite(fw["row_sum"]))
    assert np.all(fw["row_sum"][has] >= 1.0)
    for key in ("d_x", "d_k", "d_v"):
        assert np.all(np.isfinite(bw[key]))


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("model", MODELS)
def test_self_loop_only_rows_copy_the_value(model):
    H, D = 2, 4
    g = tiny_graph("selfloop", n=10)
    t, d_out = make_inputs(model, g.n, H, D, seed=4)
    fw, bw = run_oracle(layer_for(model, H, D), g, t, d_out)
    val = {"gt": t.get("v"), "gatv2": t.get("k")}.get(model, t["x"])
    np.testing.assert_allclose(fw["out"], val, rtol=1e-14)
    np.testing.assert_allclose(fw["row_sum"], 1.0)
    np.testing.assert_allclose(bw["ds"], 0.0, atol=1e-15)
    if model == "gt":
        np.testing.assert_allclose(bw["d_v"], d_out, rtol=1e-14)
        assert np.all(bw["d_x"] == 0) and np.all(bw["d_k"] == 0)
    elif model == "gatv2":
        np.testing.assert_allclose(bw["d_k"], d_out, rtol=1e-14)
        assert np.all(bw["d_x"] == 0) and np.all(bw["d_a_l"] == 0)
    else:
        np.testing.assert_allclose(bw["d_x"], d_out, rtol=1e-12, atol=1e-14)


def test_zero_query_gives_neighbourhood_mean():
    H, D = 2, 4
    g = tiny_graph("dups", seed=2, n=15)
    t, d_out = make_inputs("gt", g.n, H, D, seed=4)
    t["x"][:] = 0
    fw, _ = run_oracle(layer_for("gt", H, D), g, t, d_out)
    deg = g.degrees()
    for i in range(g.n):
        nb = g.indices[g.indptr[i]:g.indptr[i + 1]]
        if deg[i]:
            np.testing.assert_allclose(fw["out"][i], t["v"][nb].mean(0), rtol=1e-13, atol=1e-14)
            np.testing.assert_allclose(fw["row_max"][i], 0.0)
            np.testing.assert_allclose(fw["row_sum"][i], deg[i])


def test_agnn_beta_zero_and_equal_features_give_uniform_attention():
    H, D = 1, 4
    g = tiny_graph("hub", seed=2, n=15)
    t, d_out = make_inputs("agnn", g.n, H, D, seed=4)
    deg = g.degrees()
    rows = g.rows_of_edges()
    fw, _ = run_oracle(oracle.Layer("agnn", H, D, scale=0.0), g, t, d_out)
    np.testing.assert_allclose(fw["p"][:, 0], 1.0 / deg[rows], rtol=1e-13)
    t["x"][:] = np.array([0.5, -2.0, 1.0, 3.0])
    fw, bw = run_oracle(oracle.Layer("agnn", H, D, scale=2.5), g, t, d_out)
    np.testing.assert_allclose(fw["p"][:, 0], 1.0 / deg[rows], rtol=1e-12)
    np.testing.assert_allclose(fw["row_max"][deg > 0], 2.5, rtol=1e-13)  # beta * cos = beta


def test_agnn_tiny_norm_uses_eps_clamp():
    """||h|| below eps: xhat = h / eps and the gradient through the norm vanishes (dh = g / eps)."""
    H, D = 1, 3
    g = from_edge_list(3, [0, 1, 2, 0], [0, 0, 1, 2])
    x = np.array([[[1e-20, 0, 0]], [[1.0, 2.0, 0.5]], [[0.3, -1.0, 2.0]]])
    d_out = np.random.default_rng(0).standard_normal((3, H, D))
    layer = oracle.Layer("agnn", H, D, scale=1.3, eps=1e-12)
    ref, grads = dense_layer("agnn", g.indptr, g.indices, H, D, 1.3, 0.2, 1e-12, {"x": x}, d_out)
    fw = oracle.forward(layer, g.indptr, g.indices, x=x)
    bw = oracle.backward(layer, g.indptr, g.indices, x=x, d_out=d_out)
    np.testing.assert_allclose(fw["out"], ref["out"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(bw["d_x"], grads["x"], rtol=1e-9, atol=1e-12)


def test_gat_slope_one_makes_attention_independent_of_destination_term():
    """LeakyReLU with slope 1 is the identity: p_ij = softmax_j(er_j), so d_el = 0 and da_l = 0."""
    H, D = 2, 4
    g = tiny_graph("random", seed=5, n=15)
    t, d_out = make_inputs("gat", g.n, H, D, seed=4)
    layer = oracle.Layer("gat", H, D, neg_slope=1.0)
    fw, bw = run_oracle(layer, g, t, d_out)
    er = (t["x"] * t["a_r"][None]).sum(-1)
    for i in range(g.n):
        nb = g.indices[g.indptr[i]:g.indptr[i + 1]]
        if nb.size:
            e = np.exp(er[nb] - er[nb].max(0))
            np.testing.assert_allclose(fw["p"][g.indptr[i]:g.indptr[i + 1]], e / e.sum(0), rtol=1e-12)
    np.testing.assert_allclose(bw["d_a_l"], 0.0, atol=1e-13)


def test_gat_leaky_relu_derivative_at_both_signs():
    """One destination, two sources with z of opposite sign: hand-computed d_el through each branch."""
    H, D = 1, 1
    g = from_edge_list(3, [1, 2], [0, 0])
    x = np.array([[[0.0]], [[2.0]], [[-3.0]]])
    a_l, a_r = np.array([[1.0]]), np.array([[1.0]])
    d_out = np.array([[[1.0]], [[0.0]], [[0.0]]])
    layer = oracle.Layer("gat", H, D, neg_slope=0.1)
    fw = oracle.forward(layer, g.indptr, g.indices, x=x, a_l=a_l, a_r=a_r, want_p=True)
    s = np.array([2.0, -0.3])
    p = np.exp(s - s.max()) / np.exp(s - s.max()).sum()
    np.testing.assert_allclose(fw["p"][:, 0], p, rtol=1e-14)
    bw = oracle.backward(layer, g.indptr, g.indices, x=x, a_l=a_l, a_r=a_r, d_out=d_out, want_ds=True)
    dP = np.array([2.0, -3.0])
    dS = p * (dP - (p * dP).sum())
    np.testing.assert_allclose(bw["ds"][:, 0], dS, rtol=1e-13)
    dz = dS * np.array([1.0, 0.1])
    # dX_0 = d_el_0 * a_l ; dX_1 = p_1*dO_0 + d_er_1 * a_r ; dX_2 = p_2*dO_0 + d_er_2 * a_r
    np.testing.assert_allclose(bw["d_x"].ravel(), [dz.sum(), p[0] + dz[0], p[1] + dz[1]], rtol=1e-13)


def test_gatv2_slope_one_is_gat_with_one_attention_vector():
    """LeakyReLU with slope 1 is the identity, so a.(x_i + k_j) = a.x_i + a.k_j: with x = k = Wh the layer is
    GAT with a_l = a_r = a (also slope 1), and the gradients add up accordingly."""
    H, D = 2, 4
    g = tiny_graph("hub", seed=5, n=15)
    t, d_out = make_inputs("gat", g.n, H, D, seed=4)
    gat = run_oracle(oracle.Layer("gat", H, D, neg_slope=1.0), g, dict(t, a_r=t["a_l"]), d_out)
    v2 = run_oracle(oracle.Layer("gatv2", H, D, neg_slope=1.0), g, {"x": t["x"], "k": t["x"], "a_l": t["a_l"]}, d_out)
    np.testing.assert_allclose(v2[0]["out"], gat[0]["out"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(v2[0]["p"], gat[0]["p"], rtol=1e-12)
    np.testing.assert_allclose(v2[1]["d_x"] + v2[1]["d_k"], gat[1]["d_x"], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(v2[1]["d_a_l"], gat[1]["d_a_l"] + gat[1]["d_a_r"], rtol=1e-10, atol=1e-13)


def test_gatv2_ranking_depends_on_the_destination():
    """The property the variant exists for: two destinations can rank the same two sources differently
    (with GAT's separable score they cannot).  One head, D = 2, hand-computed scores."""
    H, D = 1, 2
    g = from_edge_list(4, [2, 3, 2, 3], [0, 0, 1, 1])  # destinations 0 and 1, sources 2 and 3
    x = np.array([[[2.0, -2.0]], [[-2.0, 2.0]], [[0.0, 0.0]], [[0.0, 0.0]]])
    k = np.array([[[0.0, 0.0]], [[0.0, 0.0]], [[1.0, 0.0]], [[0.0, 1.0]]])
    a = np.array([[1.0, 1.0]])
    layer = oracle.Layer("gatv2", H, D, neg_slope=0.5)
    fw = oracle.forward(layer, g.indptr, g.indices, x=x, k=k, a_l=a, want_p=True)
    lrelu = lambda z: np.where(z > 0, z, 0.5 * z)
    s = np.array([[lrelu(x[i, 0] + k[j, 0]).sum() for j in (2, 3)] for i in (0, 1)])  # [[2.0, 1.5], [1.5, 2.0]]
    np.testing.assert_allclose(s, [[2.0, 1.5], [1.5, 2.0]])
    p = np.exp(s) / np.exp(s).sum(1, keepdims=True)
    np.testing.assert_allclose(fw["p"][:, 0], p.ravel(), rtol=1e-14)
    assert fw["p"][0, 0] > fw["p"][1, 0] and fw["p"][2, 0] < fw["p"][3, 0]


# ---------------------------------------------------------------- additive edge term in the score
@pytest.mark.parametrize("model", MODELS)
@pytest.mark.parametrize("graph", ["random", "hub", "selfloop"])
def test_edge_bias_matches_dense_masked_attention(model, graph):
    H, D = 2, 4
    g = tiny_graph(graph, seed=3, n=17)
    t, d_out = make_inputs(model, g.n, H, D, seed=11)
    t["edge_bias"] = np.random.default_rng(7).standard_normal((g.nnz, H))
    layer = layer_for(model, H, D)
    fw, bw = run_oracle(layer, g, t, d_out)
    ref, grads = dense_layer(model, g.indptr, g.indices, H, D, layer.scale, layer.neg_slope, layer.eps, t, d_out)
    np.testing.assert_allclose(fw["out"], ref["out"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(bw["d_x"], grads["x"], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(bw["ds"], grads["edge_bias"], rtol=1e-9, atol=1e-12)
    if model in ("gt", "gatv2"):
        np.testing.assert_allclose(bw["d_k"], grads["k"], rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("graph", ["dups", "unsorted"])
def test_edge_bias_gradient_by_central_differences(graph):
    """Graphs the dense route cannot hold (repeated edges carry separate bias entries)."""
    H, D = 2, 3
    g = tiny_graph(graph, seed=2, n=14)
    t, d_out = make_inputs("gt", g.n, H, D, seed=23)
    t["edge_bias"] = np.random.default_rng(8).standard_normal((g.nnz, H))
    layer = layer_for("gt", H, D)
    _, bw = run_oracle(layer, g, t, d_out)
    step = 1e-6
    flat = t["edge_bias"].reshape(-1)
    for idx in np.random.default_rng(0).choice(flat.size, size=min(flat.size, 40), replace=False):
        keep = flat[idx]
        flat[idx] = keep + step
        up = _loss(layer, g, t, d_out)
        flat[idx] = keep - step
        dn = _loss(layer, g, t, d_out)
        flat[idx] = keep
        an = bw["ds"].reshape(-1)[idx]
        assert abs((up - dn) / (2 * step) - an) <= 2e-7 + 2e-6 * abs(an)


def test_edge_bias_closed_forms():
    """A bias that is constant along a row shifts the row's scores and changes nothing; with q = 0 the
    attention is softmax of the bias alone, i.e. p_ij = w_ij / sum_j w_ij for bias = log w."""
    H, D = 2, 4
    g = tiny_graph("dups", seed=2, n=15)
    t, d_out = make_inputs("gt", g.n, H, D, seed=4)
    layer = layer_for("gt", H, D)
    rows = g.rows_of_edges()
    base, _ = run_oracle(layer, g, t, d_out)
    per_row = np.random.default_rng(1).standard_normal((g.n, H))
    shifted, _ = run_oracle(layer, g, dict(t, edge_bias=per_row[rows]), d_out)
    np.testing.assert_allclose(shifted["out"], base["out"], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(shifted["p"], base["p"], rtol=1e-11)
    wgt = np.random.default_rng(2).uniform(0.1, 3.0, size=(g.nnz, H))
    t0 = dict(t, x=np.zeros_like(t["x"]), edge_bias=np.log(wgt))
    fw, _ = run_oracle(layer, g, t0, d_out)
    for h in range(H):
        tot = np.bincount(rows, weights=wgt[:, h], minlength=g.n)
        np.testing.assert_allclose(fw["p"][:, h], wgt[:, h] / tot[rows], rtol=1e-12)


# ---------------------------------------------------------------- row-subset mode used for sampled checks
@pytest.mark.parametrize("model", MODELS)
def test_row_subset_is_consistent_with_full_run(model):
    H, D = 2, 4
    g = tiny_graph("hub", seed=12, n=30)
    t, d_out = make_inputs(model, g.n, H, D, seed=4)
    layer = layer_for(model, H, D)
    fw, bw = run_oracle(layer, g, t, d_out)
    sample = np.array([5, 7, 11])
    rows = g.rows_of_edges()
    need = np.union1d(sample, rows[np.isin(g.indices, sample)])  # rows that touch a sampled node
    kw = dict(x=t["x"], k=t.get("k"), v=t.get("v"), a_l=t.get("a_l"), a_r=t.get("a_r"))
    fs = oracle.forward(layer, g.indptr, g.indices, rows=sample, **kw)
    np.testing.assert_array_equal(fs["out"][sample], fw["out"][sample])
    bs = oracle.backward(layer, g.indptr, g.indices, d_out=d_out, rows=need, **kw)
    for key in ("d_x", "d_k", "d_v"):
        if key in bw:
            np.testing.assert_allclose(bs[key][sample], bw[key][sample], rtol=1e-12, atol=1e-14)
