"""End-to-end training step of a small attention-GNN model on a synthetic workload graph: torch Linear
projections, ReLU and the optimiser around the fused graph convolutions of this library (the shape of the
paper's end-to-end comparison, Sec. 5.3: forward + backward + update of a few layers on one graph).

    python e2e_step.py --workload cfg3 --model gat --layers 2 --steps 20

Prints one JSON line: milliseconds per training step and the share spent inside the fused kernels.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--model", default="gt", choices=["gt", "gat", "gatv2", "agnn"])
    ap.add_argument("--layers", type=int, default=2)
    ap.add_argument("--hidden", type=int, default=128, help="features per layer (heads x head width)")
    ap.add_argument("--heads", type=int, default=8)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    args = ap.parse_args()

    import torch
    from torch import nn
    import paper_2411_16127_amd as dfgnn
    from paper_2411_16127_amd.nn import AGNNConv, GATConv, GATv2Conv, GTConv
    from dfgnn_synth import make_workload
    from dfgnn_synth.workloads import make_graph

    w = make_workload(args.workload)
    graph = make_graph(w)
    g = dfgnn.Graph(graph.indptr, graph.indices)
    H, D = args.heads, args.hidden // args.heads
    torch.manual_seed(w.seed)

    class Net(nn.Module):
        def __init__(self):
            super().__init__()
            self.inp = nn.Linear(args.hidden, args.hidden)
            mk = {"gt": lambda: GTConv(args.hidden, D, H), "gat": lambda: GATConv(args.hidden, D, H),
                  "gatv2": lambda: GATv2Conv(args.hidden, D, H), "agnn": lambda: AGNNConv()}[args.model]
            self.convs = nn.ModuleList([mk() for _ in range(args.layers)])
            self.out = nn.Linear(args.hidden, 16)

        def forward(self, x):
            h = torch.relu(self.inp(x))
            for conv in self.convs:
                h = h.view(-1, H, D) if args.model == "agnn" else h
                h = torch.relu(conv(g, h).flatten(1))
            return self.out(h)

    net = Net().cuda()
    opt = torch.optim.Adam(net.parameters(), lr=1e-3)
    x = torch.randn(graph.n, args.hidden, device="cuda")
    y = torch.randint(0, 16, (graph.n,), device="cuda")
    loss_fn = nn.CrossEntropyLoss()

    def step():
        opt.zero_grad(set_to_none=True)
        loss = loss_fn(net(x), y)
        loss.backward()
        opt.step()
        return loss

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps

    dfgnn.timing_enable(True)  # kernel time of the fused layers in a second run of the same steps
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    kern = dfgnn.timing_collect()
    dfgnn.timing_enable(False)
    fused_ms = sum(t for t, _ in kern.values()) / args.steps
    print(json.dumps({"workload": w.name, "N": graph.n, "E": graph.nnz, "model": args.model, "layers": args.layers,
                      "hidden": args.hidden, "heads": H, "ms_per_training_step": round(ms, 4),
                      "fused_kernels_ms_per_step": round(fused_ms, 4), "fused_share": round(fused_ms / ms, 3),
                      "final_loss": round(float(loss.detach()), 4)}))
    g.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
