"""torch.autograd wrapper of the fused layer: the graph-convolution call a model's nn.Module makes
(the "graph convolution API" of Sec. 3).  Argument marshalling only: forward and backward run in
libdfgnn through the C ABI; saved tensors are the inputs, the output and the softmax statistics."""
from __future__ import annotations

import torch

from .binding import Graph, Layer, dtype_name


class _FusedConv(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph: Graph, layer: Layer, x, k, v, a_l, a_r, edge_bias=None):
        x, k, v, edge_bias = (None if t is None else t.contiguous() for t in (x, k, v, edge_bias))
        out, row_max, row_sum = graph.forward(layer, x, k, v, a_l, a_r, edge_bias=edge_bias)
        ctx.graph, ctx.layer = graph, layer
        ctx.save_for_backward(*(t for t in (x, k, v, a_l, a_r, edge_bias, out, row_max, row_sum) if t is not None))
        ctx.has = tuple(t is not None for t in (x, k, v, a_l, a_r, edge_bias))
        ctx.bias_grad = edge_bias is not None and edge_bias.requires_grad
        return out

    @staticmethod
    def backward(ctx, d_out):
        saved = list(ctx.saved_tensors)
        x, k, v, a_l, a_r, edge_bias = (saved.pop(0) if h else None for h in ctx.has)
        out, row_max, row_sum = saved
        g = ctx.graph.backward(ctx.layer, x, k, v, a_l, a_r, out, row_max, row_sum, d_out.contiguous(),
                               edge_bias=edge_bias, want_d_edge_bias=ctx.bias_grad)
        return (None, None, g["d_x"], g.get("d_k"), g.get("d_v"), g.get("d_a_l"), g.get("d_a_r"), g.get("d_edge_bias"))


def _kernel_width(D: int, dtype) -> int:
    """Head width the kernels accept: a power-of-two number of 16-byte lanes."""
    per_lane = 4 if dtype == torch.float32 else 8
    lanes = 1
    while lanes * per_lane < D:
        lanes *= 2
    return lanes * per_lane


def _pad(t, width: int):
    """Zero-pads the features of every head to `width`.  Zero features change no score of any of the models
    (dot products, norms and a.LeakyReLU(0) terms are unaffected) and aggregate to zero, so the wrappers
    pad odd head widths, call the kernels, and cut the padding off the result; torch differentiates both."""
    return t if t.shape[-1] == width else torch.nn.functional.pad(t, (0, width - t.shape[-1]))


def gt_conv(graph: Graph, q, k, v, scale=None, edge_bias=None):
    """Graph-transformer convolution: softmax over in-neighbours of scale * q_i.k_j (+ edge_bias [E,H], fp32, in
    CSR edge order, if given), applied to v.  [N,H,D]."""
    H, D = q.shape[1], q.shape[2]
    W = _kernel_width(D, q.dtype)
    layer = Layer("gt", H, W, dtype=dtype_name(q.dtype),
                  scale=float(D) ** -0.5 if scale is None else float(scale))
    return _FusedConv.apply(graph, layer, _pad(q, W), _pad(k, W), _pad(v, W), None, None, edge_bias)[..., :D]


def gat_conv(graph: Graph, wh, a_l, a_r, neg_slope: float = 0.2):
    """GAT convolution on projected features Wh [N,H,D] with attention vectors a_l, a_r [H,D] (fp32)."""
    H, D = wh.shape[1], wh.shape[2]
    W = _kernel_width(D, wh.dtype)
    layer = Layer("gat", H, W, dtype=dtype_name(wh.dtype), neg_slope=float(neg_slope))
    return _FusedConv.apply(graph, layer, _pad(wh, W), None, None, _pad(a_l, W).contiguous(),
                            _pad(a_r, W).contiguous())[..., :D]


def gatv2_conv(graph: Graph, x_dst, x_src, a, neg_slope: float = 0.2):
    """GATv2 convolution: scores sum_d a_d LeakyReLU(x_dst_i,d + x_src_j,d), applied to x_src.  x_dst, x_src:
    the two projections of the node features [N,H,D]; a [H,D] (fp32)."""
    H, D = x_dst.shape[1], x_dst.shape[2]
    W = _kernel_width(D, x_dst.dtype)
    layer = Layer("gatv2", H, W, dtype=dtype_name(x_dst.dtype), neg_slope=float(neg_slope))
    return _FusedConv.apply(graph, layer, _pad(x_dst, W), _pad(x_src, W), None, _pad(a, W).contiguous(), None)[..., :D]


class _AgnnConv(torch.autograd.Function):
    """AGNN needs the gradient of the scalar beta.  A beta that lives on the GPU (a trained parameter) is handed to
    the library as a device pointer, so neither call reads it back to the host."""

    @staticmethod
    def forward(ctx, graph: Graph, h, beta, eps: float):
        on_device = beta.is_cuda
        beta_dev = beta.detach().reshape(1).to(torch.float32).contiguous() if on_device else None
        layer = Layer("agnn", h.shape[1], h.shape[2], dtype=dtype_name(h.dtype),
                      scale=1.0 if on_device else float(beta.detach()), eps=eps)
        h = h.contiguous()
        out, row_max, row_sum = graph.forward(layer, h, a_l=beta_dev)
        ctx.graph, ctx.layer = graph, layer
        ctx.save_for_backward(h, out, row_max, row_sum, beta, *((beta_dev,) if on_device else ()))
        return out

    @staticmethod
    def backward(ctx, d_out):
        h, out, row_max, row_sum, beta, *rest = ctx.saved_tensors
        g = ctx.graph.backward(ctx.layer, h, None, None, rest[0] if rest else None, None, out, row_max, row_sum,
                               d_out.contiguous())
        return None, g["d_x"], g["d_scale"].to(dtype=beta.dtype, device=beta.device).reshape(beta.shape), None


def agnn_conv(graph: Graph, h, beta, eps: float = 1e-12):
    """AGNN convolution: softmax of beta * cos(h_i, h_j), applied to h.  beta: 0-d or 1-element tensor."""
    D = h.shape[2]
    return _AgnnConv.apply(graph, _pad(h, _kernel_width(D, h.dtype)), beta, eps)[..., :D]
