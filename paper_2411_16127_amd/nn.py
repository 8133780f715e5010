"""torch.nn modules around the fused layer, in the shape of the usual graph-convolution classes: the dense
projections are ordinary torch Linear layers (they are outside the fused kernel, Eq. 1 starts from Q, K, V),
the attention, edge softmax and aggregation run in libdfgnn through the autograd wrappers."""
from __future__ import annotations

import torch
from torch import nn

from .autograd import agnn_conv, gat_conv, gatv2_conv, gt_conv
from .binding import Graph


class GTConv(nn.Module):
    """Graph-transformer convolution: per head, softmax_j(q_i.k_j / sqrt(D)) over in-neighbours, applied to v.

    The three projections are one batched product: weight [3, in, H*D], result [3, N, H*D], whose slices are
    the contiguous Q, K, V tensors the fused layer takes (one GEMM launch instead of three, and no copies)."""

    def __init__(self, in_feats: int, out_feats: int, num_heads: int, bias: bool = True):
        super().__init__()
        self.num_heads, self.out_feats = num_heads, out_feats
        width = num_heads * out_feats
        self.w_qkv = nn.Parameter(torch.empty(3, in_feats, width))
        self.b_qkv = nn.Parameter(torch.zeros(3, 1, width)) if bias else None
        bound = in_feats ** -0.5  # the default range of nn.Linear
        nn.init.uniform_(self.w_qkv, -bound, bound)
        if bias:
            nn.init.uniform_(self.b_qkv, -bound, bound)

    def forward(self, graph: Graph, feat, edge_bias=None):
        x3 = feat.unsqueeze(0).expand(3, -1, -1)
        qkv = torch.bmm(x3, self.w_qkv) if self.b_qkv is None else torch.baddbmm(self.b_qkv, x3, self.w_qkv)
        shape = (-1, self.num_heads, self.out_feats)
        return gt_conv(graph, qkv[0].view(shape), qkv[1].view(shape), qkv[2].view(shape), edge_bias=edge_bias)


class GATConv(nn.Module):
    """GAT convolution: scores LeakyReLU(a_l.Wh_i + a_r.Wh_j), aggregated value Wh_j."""

    def __init__(self, in_feats: int, out_feats: int, num_heads: int, negative_slope: float = 0.2):
        super().__init__()
        self.num_heads, self.out_feats, self.negative_slope = num_heads, out_feats, negative_slope
        self.fc = nn.Linear(in_feats, num_heads * out_feats, bias=False)
        self.attn_l = nn.Parameter(torch.empty(num_heads, out_feats))
        self.attn_r = nn.Parameter(torch.empty(num_heads, out_feats))
        gain = nn.init.calculate_gain("relu")
        nn.init.xavier_normal_(self.attn_l, gain=gain)
        nn.init.xavier_normal_(self.attn_r, gain=gain)

    def forward(self, graph: Graph, feat):
        wh = self.fc(feat).view(-1, self.num_heads, self.out_feats)
        return gat_conv(graph, wh, self.attn_l.float(), self.attn_r.float(), self.negative_slope)


class GATv2Conv(nn.Module):
    """GATv2 convolution: scores a.LeakyReLU(W_dst h_i + W_src h_j), aggregated value W_src h_j."""

    def __init__(self, in_feats: int, out_feats: int, num_heads: int, negative_slope: float = 0.2,
                 share_weights: bool = False):
        super().__init__()
        self.num_heads, self.out_feats, self.negative_slope = num_heads, out_feats, negative_slope
        self.fc_src = nn.Linear(in_feats, num_heads * out_feats, bias=True)
        self.fc_dst = self.fc_src if share_weights else nn.Linear(in_feats, num_heads * out_feats, bias=True)
        self.attn = nn.Parameter(torch.empty(num_heads, out_feats))
        nn.init.xavier_normal_(self.attn, gain=nn.init.calculate_gain("relu"))

    def forward(self, graph: Graph, feat):
        shape = (-1, self.num_heads, self.out_feats)
        return gatv2_conv(graph, self.fc_dst(feat).view(shape), self.fc_src(feat).view(shape), self.attn.float(),
                          self.negative_slope)


class AGNNConv(nn.Module):
    """AGNN propagation: scores beta * cos(h_i, h_j) per head, aggregated value h_j; beta is learnable."""

    def __init__(self, init_beta: float = 1.0, learn_beta: bool = True, eps: float = 1e-12):
        super().__init__()
        self.eps = eps
        beta = torch.tensor(float(init_beta))
        self.beta = nn.Parameter(beta) if learn_beta else None
        if not learn_beta:
            self.register_buffer("fixed_beta", beta)

    def forward(self, graph: Graph, feat):
        h = feat if feat.dim() == 3 else feat.unsqueeze(1)
        beta = self.beta if self.beta is not None else self.fixed_beta
        out = agnn_conv(graph, h, beta, self.eps)
        return out if feat.dim() == 3 else out.squeeze(1)
