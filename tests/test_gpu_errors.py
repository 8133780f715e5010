"""Error paths and degenerate inputs of the C ABI, forced from the host (every kernel that does run stays in bounds)."""
import numpy as np
import pytest

import paper_2411_16127_amd as dfgnn
from dfgnn_synth import tiny_graph

pytestmark = pytest.mark.gpu

EINVAL, EUNSUPPORTED, EWORKSPACE = 1, 2, 3


def raw_create(indptr, indices, n=None, e=None, meta_slack=0, misalign=0):
    import torch
    ip = torch.tensor(indptr, dtype=torch.int32, device="cuda")
    ix = torch.tensor(indices, dtype=torch.int32, device="cuda") if len(indices) else torch.zeros(1, dtype=torch.int32, device="cuda")
    n = len(indptr) - 1 if n is None else n
    e = len(indices) if e is None else e
    mb, sb = dfgnn.graph_meta_bytes(n, e)
    meta = torch.empty(mb + 512, dtype=torch.uint8, device="cuda")
    scratch = torch.empty(sb + 512, dtype=torch.uint8, device="cuda")
    h = dfgnn.graph_create(n, e, ip, ix, None, meta.data_ptr() + misalign, mb + meta_slack, scratch, sb)
    return h, (ip, ix, meta, scratch)


@pytest.mark.parametrize("indptr,indices", [
    ([1, 2, 3], [0, 1, 0]),        # indptr[0] != 0
    ([0, 2, 1, 3], [0, 1, 2]),     # decreasing
    ([0, 1, 2], [0, 1, 0]),        # indptr[N] != E
    ([0, 1, 2], [0, 7]),           # index out of range
    ([0, 1, 2], [0, -1]),          # negative index
])
def test_malformed_csr_is_rejected(indptr, indices):
    with pytest.raises(dfgnn.DfgnnError) as e:
        raw_create(indptr, indices)
    assert e.value.status == EINVAL and "malformed CSR" in str(e.value)


def test_small_or_misaligned_buffers_are_rejected():
    g = tiny_graph("random", seed=1, n=30)
    with pytest.raises(dfgnn.DfgnnError) as e:
        raw_create(g.indptr.tolist(), g.indices.tolist(), meta_slack=-256)
    assert e.value.status == EWORKSPACE
    with pytest.raises(dfgnn.DfgnnError) as e:
        raw_create(g.indptr.tolist(), g.indices.tolist(), misalign=4)
    assert e.value.status == EUNSUPPORTED
    h, keep = raw_create(g.indptr.tolist(), g.indices.tolist())
    dfgnn.graph_destroy(h)


def test_layer_argument_checks():
    import torch
    graph = tiny_graph("hub", seed=1, n=40)
    g = dfgnn.Graph(graph.indptr, graph.indices, dfgnn.SchedParams(8, 4))
    N = graph.n

    def call(layer, x, k=None, v=None, a_l=None, a_r=None, ws_bytes=None, x_off=0):
        out = torch.empty(N * layer.H * layer.D, dtype=torch.float32, device="cuda")
        st = torch.empty(N * layer.H, dtype=torch.float32, device="cuda")
        st2 = torch.empty_like(st)
        ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
        xp = None if x is None else x.data_ptr() + x_off
        dfgnn.forward(g.handle, layer, xp, k, v, a_l, a_r, out, st, st2, ws, ws.numel() if ws_bytes is None else ws_bytes)

    def status(**kw):
        with pytest.raises(dfgnn.DfgnnError) as e:
            call(**kw)
        return e.value.status

    x = torch.zeros(N * 64 + 16, dtype=torch.float32, device="cuda")
    gt = dfgnn.Layer("gt", 1, 64)
    assert status(layer=dfgnn.Layer("gt", 1, 6), x=x, k=x, v=x) == EUNSUPPORTED      # head not a multiple of 16 bytes
    assert status(layer=dfgnn.Layer("gt", 1, 12), x=x, k=x, v=x) == EUNSUPPORTED     # D/4 not a power of two
    assert status(layer=dfgnn.Layer("gt", 1, 512), x=x, k=x, v=x) == EUNSUPPORTED    # one head wider than a wavefront
    assert status(layer=dfgnn.Layer("gt", 0, 64), x=x, k=x, v=x) == EINVAL
    assert status(layer=gt, x=x, k=None, v=x) == EINVAL                                # GT needs k
    assert status(layer=gt, x=x, k=x, v=x, a_l=x) == EINVAL                            # a_l only for GAT
    assert status(layer=dfgnn.Layer("gat", 1, 64), x=x) == EINVAL                      # GAT needs a_l, a_r
    assert status(layer=dfgnn.Layer("agnn", 1, 64), x=x, k=x) == EINVAL                # k only for GT
    assert status(layer=dfgnn.Layer("agnn", 1, 64, eps=0.0), x=x) == EINVAL
    assert status(layer=gt, x=x, k=x, v=x, ws_bytes=64) == EWORKSPACE                  # super rows need partials
    assert status(layer=gt, x=x, k=x, v=x, x_off=4) == EUNSUPPORTED                    # 16-byte alignment
    assert status(layer=gt, x=None, k=x, v=x) == EINVAL
    with pytest.raises(dfgnn.DfgnnError) as e:
        dfgnn.graph_query(g.handle, 99)
    assert e.value.status == EINVAL
    call(layer=gt, x=x, k=x, v=x)  # the well-formed call still works afterwards
    torch.cuda.synchronize()
    assert dfgnn.last_error() == ""
    g.close()


@pytest.mark.parametrize("model", ["gt", "gat", "agnn", "gatv2"])
def test_graph_without_edges_and_empty_graph(model):
    import torch
    H, D = 2, 8
    L = dfgnn.Layer(model, H, D, scale=0.7)
    for n in (0, 9):
        g = dfgnn.Graph(np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32))
        x = torch.randn(n, H, D, device="cuda")
        kv = (x.clone(), x.clone()) if model == "gt" else ((x.clone(), None) if model == "gatv2" else (None, None))
        att = (torch.randn(H, D, device="cuda"), torch.randn(H, D, device="cuda")) if model == "gat" else (
            (torch.randn(H, D, device="cuda"), None) if model == "gatv2" else (None, None))
        out, rmax, rsum = g.forward(L, x, kv[0], kv[1], att[0], att[1])
        grads = g.backward(L, x, kv[0], kv[1], att[0], att[1], out, rmax, rsum, torch.randn_like(x))
        torch.cuda.synchronize()
        assert torch.all(out == 0) and torch.all(rsum == 0) and torch.all(torch.isneginf(rmax))
        for key, val in grads.items():
            assert torch.all(val == 0), key
        g.close()
