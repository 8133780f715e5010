"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI binding, run the CPU
oracle on the same seeded inputs, compare element by element."""
import numpy as np

import oracle
import paper_2411_16127_amd as dfgnn

# fp32: |gpu - ref| <= 1e-5 + 1e-4 |ref|.  bf16 tensors: 2e-2 relative plus max(2e-2 * rms(ref), 1e-5) absolute
# (the stated tolerance has no absolute term).
F32_RTOL, F32_ATOL = 1e-4, 1e-5
BF16_RTOL = 2e-2


def to_device(arr, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(arr)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


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


def run_oracle(graph, w, feats, rows=None, backward_rows=None):
    L = oracle_layer(w)
    kw = dict(x=feats["q"] if w.model == "gt" else feats["feat"], k=feats.get("k"), v=feats.get("v"),
              a_l=feats.get("a_l"), a_r=feats.get("a_r"), edge_bias=feats.get("edge_bias"))
    kw = {k_: (None if v_ is None else np.asarray(v_, dtype=np.float64)) for k_, v_ in kw.items()}
    fw = oracle.forward(L, graph.indptr, graph.indices, rows=rows, **kw)
    bw = oracle.backward(L, graph.indptr, graph.indices, d_out=np.asarray(feats["d_out"], dtype=np.float64),
                         rows=backward_rows, want_ds="edge_bias" in feats, **kw)
    ref = dict(fw)
    ref.update(bw)
    if "ds" in ref:
        ref["d_edge_bias"] = ref.pop("ds")
    if "d_scale" in ref:
        ref["d_scale"] = np.array([ref["d_scale"]])
    return ref


def _rms(ref):
    fin = ref[np.isfinite(ref)]
    return float(np.sqrt(np.mean(np.square(fin)))) if fin.size else 0.0


def tolerance(name, ref, dtype):
    """(rtol, atol, floor): bound = atol + rtol * max(|ref|, floor).

    Node tensors and statistics of fp32 layers: the stated 1e-4 / 1e-5, element by element.
    Parameter gradients (d_a_l, d_a_r, d_scale) are sums of signed terms over all nodes and edges; their
    fp32 error scales with the size of the terms, not of the (partly cancelled) result, so the relative
    part is taken against the rms of the gradient vector when an element is smaller than that.
    bf16 layers: 2e-2 relative plus 2e-2 * rms(ref) absolute, the absolute part never below the fp32 one:
    where the exact result is zero throughout (dS = 0 when every row has a single edge) the computed one is
    the fp32 rounding of terms that cancel.
    """
    if dtype == "bf16":
        return BF16_RTOL, max(BF16_RTOL * _rms(ref), F32_ATOL), 0.0
    if name in ("d_a_l", "d_a_r", "d_scale"):
        return F32_RTOL, F32_ATOL, _rms(ref)
    return F32_RTOL, F32_ATOL, 0.0


def assert_close(name, got, ref, dtype, rows=None, tol=None):
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    if rows is not None:
        got, ref = got[rows], ref[rows]
    rtol, atol, floor = tol or tolerance(name, ref, dtype)
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
    names = keys or [k for k in ("out", "row_max", "row_sum", "d_x", "d_k", "d_v", "d_a_l", "d_a_r", "d_scale",
                                 "d_edge_bias") if k in ref]
    for name in names:
        per_node = name in ("out", "row_max", "row_sum", "d_x", "d_k", "d_v")
        assert_close(name, res[name], ref[name], w.dtype, rows if per_node else None, tol)
