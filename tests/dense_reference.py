"""Dense masked-attention formulation of the models in CPU torch float64 + autograd.

Used only to pin the CPU oracle: it is a different route to the same numbers (dense N x N score
matrix, library softmax, library autograd) and shares nothing with the oracle or the HIP path.
Cannot represent duplicate edges; callers pass duplicate-free graphs.
"""
import numpy as np
import torch


def dense_layer(model, indptr, indices, H, D, scale, neg_slope, eps, tensors, d_out):
    """tensors: dict of numpy arrays (x, k, v, a_l, a_r as applicable; optional edge_bias [nnz, H] in CSR
    edge order, added to the scores).  Returns (outputs, grads)."""
    n = len(indptr) - 1
    mask = torch.zeros(n, n, dtype=torch.bool)  # mask[i, j] = edge i <- j
    for i in range(n):
        for t in range(indptr[i], indptr[i + 1]):
            assert not mask[i, indices[t]], "dense reference cannot hold duplicate edges"
            mask[i, indices[t]] = True
    t = {k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in tensors.items()}
    beta = torch.tensor(float(scale), dtype=torch.float64, requires_grad=True)
    if model == "gt":
        s = scale * torch.einsum("ihd,jhd->hij", t["x"], t["k"])
        val = t["v"]
    elif model == "gat":
        el = (t["x"] * t["a_l"][None]).sum(-1)  # [n, H]
        er = (t["x"] * t["a_r"][None]).sum(-1)
        z = el.t()[:, :, None] + er.t()[:, None, :]  # [H, i, j]
        s = torch.nn.functional.leaky_relu(z, neg_slope)
        val = t["x"]
    elif model == "gatv2":
        z = t["x"].permute(1, 0, 2)[:, :, None, :] + t["k"].permute(1, 0, 2)[:, None, :, :]  # [H, i, j, D]
        s = (torch.nn.functional.leaky_relu(z, neg_slope) * t["a_l"][:, None, None, :]).sum(-1)
        val = t["k"]
    elif model == "agnn":
        nrm = torch.clamp(torch.linalg.vector_norm(t["x"], dim=-1, keepdim=True), min=eps)
        xh = t["x"] / nrm
        s = beta * torch.einsum("ihd,jhd->hij", xh, xh)
        val = t["x"]
    else:
        raise ValueError(model)
    if "edge_bias" in t:  # scatter the per-edge term into the dense [H, i, j] score matrix
        rows_of = torch.tensor(np.repeat(np.arange(n), np.diff(indptr)), dtype=torch.long)
        cols_of = torch.tensor(np.asarray(indices), dtype=torch.long)
        dense_b = torch.zeros(H, n, n, dtype=torch.float64)
        dense_b = dense_b.index_put((torch.arange(H)[:, None], rows_of[None, :], cols_of[None, :]), t["edge_bias"].t())
        s = s + dense_b
    has = mask.any(dim=1)
    s = s.masked_fill(~mask[None], float("-inf"))
    s_safe = torch.where(has[None, :, None], s, torch.zeros_like(s))
    p = torch.softmax(s_safe, dim=-1)
    p = torch.where(mask[None] & has[None, :, None], p, torch.zeros_like(p))
    out = torch.einsum("hij,jhd->ihd", p, val)
    row_max = torch.where(has[None], s.max(dim=-1).values, torch.full((H, n), float("-inf"), dtype=torch.float64))
    loss = (out * torch.tensor(np.asarray(d_out, dtype=np.float64))).sum()
    loss.backward()
    grads = {k: (v.grad.numpy() if v.grad is not None else None) for k, v in t.items()}
    grads["beta"] = None if beta.grad is None else float(beta.grad)
    return {"out": out.detach().numpy(), "row_max": row_max.t().detach().numpy(), "p": p.detach().numpy()}, grads
