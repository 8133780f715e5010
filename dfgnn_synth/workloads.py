"""The five benchmark workloads (graph + layer shape + seeded features).

Each workload stands in for a group of the evaluated datasets (dataset table,
Sec. 5.1; model settings: feature dimension 128, batch size 1024): the graphs
have the same node/edge counts and degree skew, the features are i.i.d.
normal.  Seeds: graph = 1000 + workload number, features = that + 1 (one
sub-stream per tensor), upstream gradient = that + 2.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

from . import graphs as G


@dataclass(frozen=True)
class Workload:
    name: str
    number: int
    model: str  # 'gt' | 'gat' | 'agnn' | 'gatv2'
    H: int
    D: int
    dtype: str  # 'f32' | 'bf16' | 'f16' (storage type of node tensors)
    scale: float  # GT: multiplies q.k ; AGNN: beta ; GAT: unused (1.0)
    neg_slope: float = 0.2
    eps: float = 1e-12
    kind: str = "chung_lu"  # graph family
    n: int = 0
    n_edges: int = 0  # non-self edges (chung_lu), uniform edges (hub)
    gamma: float = 2.5
    max_weight: float = 0.0
    n_hubs: int = 0
    hub_in_degree: int = 0
    n_graphs: int = 0
    n_min: int = 0
    n_max: int = 0
    density: float = 0.0
    stands_in_for: str = ""

    @property
    def seed(self) -> int:
        return 1000 + self.number


WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", 1, "gt", 1, 64, "f32", 1.0 / 8.0, kind="chung_lu", n=2708, n_edges=10556,
                     gamma=2.5, max_weight=170.0, stands_in_for="small citation full graph (2.7K nodes, 10K edges)"),
    "cfg2": Workload("cfg2", 2, "gt", 8, 16, "bf16", 0.25, kind="batched", n_graphs=1024, n_min=10, n_max=40,
                     density=0.3, stands_in_for="batch-graph datasets at batch size 1024"),
    "cfg3": Workload("cfg3", 3, "gat", 8, 8, "f32", 1.0, neg_slope=0.2, kind="chung_lu", n=169343,
                     n_edges=2300000, gamma=2.2, max_weight=13000.0,
                     stands_in_for="mid-size citation full graph (169K nodes)"),
    "cfg4": Workload("cfg4", 4, "agnn", 1, 64, "f32", 1.0, kind="hub", n=1000000, n_edges=8000000, n_hubs=16,
                     hub_in_degree=200000, stands_in_for="super-node full graphs, extreme hub/mean ratio"),
    "cfg5": Workload("cfg5", 5, "gt", 8, 16, "f32", 0.25, kind="chung_lu", n=2449029, n_edges=122500000 - 2449029,
                     gamma=2.1, max_weight=17000.0,
                     stands_in_for="largest super-node full graph (114M edges, max degree 21,657)"),
}


def make_workload(name: str, shrink: int = 1, **overrides) -> Workload:
    """Return a workload; shrink > 1 divides node/edge/graph counts (test-size variants)."""
    w = WORKLOADS[name]
    if shrink > 1:
        w = replace(
            w,
            n=max(w.n // shrink, 64) if w.n else 0,
            n_edges=max(w.n_edges // shrink, 128) if w.n_edges else 0,
            hub_in_degree=max(w.hub_in_degree // shrink, 32) if w.hub_in_degree else 0,
            n_graphs=max(w.n_graphs // shrink, 4) if w.n_graphs else 0,
            max_weight=max(w.max_weight / shrink ** 0.5, 16.0) if w.max_weight else 0.0,
        )
    if overrides:
        w = replace(w, **overrides)
    return w


def make_graph(w: Workload) -> G.Graph:
    if w.kind == "chung_lu":
        return G.chung_lu_graph(w.n, w.n_edges, w.gamma, w.max_weight, w.seed, self_loops=True)
    if w.kind == "hub":
        return G.hub_graph(w.n, w.n_edges, w.n_hubs, min(w.hub_in_degree, w.n - 1), w.seed)
    if w.kind == "batched":
        return G.batched_small_graphs(w.n_graphs, w.n_min, w.n_max, w.density, w.seed)
    raise ValueError(w.kind)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    out = (rounded & 0xFFFFFFFF).astype(np.uint32).view(np.float32)
    return np.where(np.isfinite(x), out, x).astype(np.float32)


def _normal(seed: int, stream: int, shape, std: float = 1.0) -> np.ndarray:
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(seed), int(stream)])))
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def make_features(w: Workload, n: int, seed: Optional[int] = None, threads: int = 4) -> Dict[str, np.ndarray]:
    """Node tensors [n, H, D] float32 (bf16 / f16 workloads: values already rounded to that type).

    GT: q, k, v;  GAT: feat (=Wh), a_l, a_r [H, D] fp32;  AGNN: feat (=h);  GATv2: feat (destination-side
    projection), k (source-side projection), a_l (= a) [H, D] fp32.
    'd_out' is the upstream gradient dL/dO.  Every tensor has its own random stream, so the values do
    not depend on `threads` (tensors are drawn concurrently).
    """
    from concurrent.futures import ThreadPoolExecutor

    s = w.seed if seed is None else seed
    shape = (n, w.H, w.D)
    if w.model == "gt":
        jobs = {"q": (s + 1, 0, shape, 1.0), "k": (s + 1, 1, shape, 1.0), "v": (s + 1, 2, shape, 1.0)}
    elif w.model == "gat":
        jobs = {"feat": (s + 1, 0, shape, 1.0), "a_l": (s + 1, 1, (w.H, w.D), 0.1), "a_r": (s + 1, 2, (w.H, w.D), 0.1)}
    elif w.model == "gatv2":
        jobs = {"feat": (s + 1, 0, shape, 1.0), "k": (s + 1, 1, shape, 1.0), "a_l": (s + 1, 2, (w.H, w.D), 0.1)}
    elif w.model == "agnn":
        jobs = {"feat": (s + 1, 0, shape, 1.0)}
    else:
        raise ValueError(w.model)
    jobs["d_out"] = (s + 2, 0, shape, 1.0)

    def draw(item):
        key, (seed_, stream, shp, std) = item
        x = _normal(seed_, stream, shp, std)
        if w.dtype == "bf16" and key in ("q", "k", "v", "feat", "d_out"):
            x = round_to_bf16(x)
        if w.dtype == "f16" and key in ("q", "k", "v", "feat", "d_out"):
            x = x.astype(np.float16).astype(np.float32)  # round to nearest even
        return key, x

    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        return dict(pool.map(draw, jobs.items()))
