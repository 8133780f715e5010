"""Seeded synthetic graph generators, CSR by destination.

Row i of the CSR lists the in-neighbours (sources j of edges i <- j) of
destination i; this is the neighbourhood N(v) that the edge softmax of
Appendix A normalises over.  All generators are deterministic functions of
their arguments (numpy SFC64 streams derived from the seed) and emit int32
arrays with sources ascending inside every row and no duplicate edges, unless
a caller of `from_edge_list` asks otherwise.

The shapes follow the dataset table of Sec. 5.1 (node and edge counts,
average / maximum degree); the real datasets are not used anywhere.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass
class Graph:
    n: int
    indptr: np.ndarray  # int32 [n + 1]
    indices: np.ndarray  # int32 [nnz], source ids
    batch_ptr: Optional[np.ndarray] = None  # int32 [n_graphs + 1] node offsets of a block-diagonal batch

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])

    def degrees(self) -> np.ndarray:
        return np.diff(self.indptr.astype(np.int64))

    def rows_of_edges(self) -> np.ndarray:
        """Destination id of every stored edge (COO expansion of indptr)."""
        return np.repeat(np.arange(self.n, dtype=np.int32), self.degrees())


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(seed), int(stream)])))


def from_edge_list(n: int, src, dst, *, sort: bool = True, dedupe: bool = False,
                   batch_ptr=None) -> Graph:
    """Build a CSR-by-destination graph from edge arrays (edge = dst <- src).

    sort=False keeps the given order of sources inside a row (rows are still
    grouped, stably); dedupe=False keeps repeated edges as separate entries.
    """
    src = np.asarray(src, dtype=np.int64).ravel()
    dst = np.asarray(dst, dtype=np.int64).ravel()
    if src.shape != dst.shape:
        raise ValueError("src and dst differ in length")
    if src.size and (src.min() < 0 or src.max() >= n or dst.min() < 0 or dst.max() >= n):
        raise ValueError("edge endpoint out of range")
    if sort:
        key = dst * n + src
        key = np.unique(key) if dedupe else np.sort(key, kind="stable")
        dst, src = key // n, key % n
    else:
        if dedupe:
            raise ValueError("dedupe requires sort=True")
        order = np.argsort(dst, kind="stable")
        dst, src = dst[order], src[order]
    counts = np.bincount(dst, minlength=n)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=indptr[1:])
    if indptr[-1] >= 2**31:
        raise ValueError("edge count does not fit int32")
    bp = None if batch_ptr is None else np.asarray(batch_ptr, dtype=np.int32)
    return Graph(int(n), indptr.astype(np.int32), src.astype(np.int32), bp)


def _add_self_loops_sorted(n: int, key: np.ndarray) -> Graph:
    """key: sorted unique dst*n+src with no self pairs -> CSR with one self-loop per node."""
    dst = key // n
    src = key - dst * n
    below = np.bincount(dst[src < dst], minlength=n)  # sources smaller than the row id
    counts = np.bincount(dst, minlength=n)
    old_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=old_ptr[1:])
    nnz = key.size + n
    indices = np.empty(nnz, dtype=np.int32)
    # an old edge at position e of row d moves right by d (loops of earlier rows) + 1 if past the loop
    pos = np.arange(key.size, dtype=np.int64) + dst + (src > dst)
    indices[pos] = src
    rows = np.arange(n, dtype=np.int64)
    indices[old_ptr[:-1] + rows + below] = rows
    indptr = old_ptr + np.arange(n + 1, dtype=np.int64)
    return Graph(int(n), indptr.astype(np.int32), indices)


def _solve_k0(n: int, n_edges: int, a: float, max_weight: float) -> float:
    """Offset k0 of the rank weights w_k ~ (k + k0)^(-a) with sum n_edges and w_0 = max_weight."""
    def w0(k0: float) -> float:
        e = 1.0 - a
        return n_edges * ((1.0 + k0) ** e - k0 ** e) / ((n + k0) ** e - k0 ** e)
    lo, hi = 1e-12, 1e12
    for _ in range(200):
        mid = (lo * hi) ** 0.5
        if w0(mid) > max_weight:
            lo = mid
        else:
            hi = mid
    return (lo * hi) ** 0.5


def chung_lu_graph(n: int, n_edges: int, gamma: float, max_weight: float, seed: int,
                   self_loops: bool = True) -> Graph:
    """Directed Chung-Lu graph with a power-law expected-degree sequence.

    Rank r in [0, n) has expected in- and out-degree w_r proportional to
    (r + k0)^(-1/(gamma-1)); k0 is solved so that sum w = n_edges and
    w_0 = max_weight.  Both endpoints of a candidate edge are drawn i.i.d.
    proportional to w (continuous inverse-CDF, floor to a rank), ranks are
    mapped to node ids through a random permutation, self pairs and repeated
    pairs are dropped, sampling repeats until at least n_edges distinct pairs
    exist and a uniformly random surplus is removed so that exactly n_edges
    remain; finally one self-loop per node is added (self_loops=True).
    """
    if not (gamma > 2.0):
        raise ValueError("gamma must exceed 2 (finite mean)")
    a = 1.0 / (gamma - 1.0)
    e = 1.0 - a
    k0 = _solve_k0(n, n_edges, a, max_weight)
    lo, hi = k0 ** e, (n + k0) ** e
    rng = _rng(seed, 0)
    perm = rng.permutation(n).astype(np.int64)

    def draw(m: int) -> np.ndarray:
        ends = []
        for _ in range(2):
            u = rng.random(m)
            x = (lo + u * (hi - lo)) ** (1.0 / e) - k0
            r = np.clip(x.astype(np.int64), 0, n - 1)
            ends.append(perm[r])
        src, dst = ends
        keep = src != dst
        return dst[keep] * n + src[keep]

    key = np.empty(0, dtype=np.int64)
    while key.size < n_edges:
        m = int((n_edges - key.size) * 1.06) + 1024
        key = np.unique(np.concatenate([key, draw(m)]))
    surplus = key.size - n_edges
    if surplus:
        mask = np.ones(key.size, dtype=bool)
        mask[rng.choice(key.size, size=surplus, replace=False)] = False
        key = key[mask]
    if self_loops:
        return _add_self_loops_sorted(n, key)
    return from_edge_list(n, key % n, key // n)


def hub_graph(n: int, n_uniform_edges: int, n_hubs: int, hub_in_degree: int, seed: int) -> Graph:
    """Uniform random directed edges plus a few destinations with huge in-degree.

    n_uniform_edges distinct (src, dst) pairs, src != dst, uniform over nodes;
    n_hubs distinct hub destinations, each receiving edges from hub_in_degree
    distinct uniformly random sources (not itself).  No self-loops are added,
    so some rows are empty.  An edge present in both parts is stored once.
    """
    rng = _rng(seed, 0)
    key = np.empty(0, dtype=np.int64)
    while key.size < n_uniform_edges:
        m = int((n_uniform_edges - key.size) * 1.02) + 1024
        src = rng.integers(0, n, size=m, dtype=np.int64)
        dst = rng.integers(0, n, size=m, dtype=np.int64)
        keep = src != dst
        key = np.unique(np.concatenate([key, dst[keep] * n + src[keep]]))
    surplus = key.size - n_uniform_edges
    if surplus:
        mask = np.ones(key.size, dtype=bool)
        mask[rng.choice(key.size, size=surplus, replace=False)] = False
        key = key[mask]
    hubs = rng.choice(n, size=n_hubs, replace=False).astype(np.int64)
    parts = [key]
    for hub in hubs:
        cand = rng.choice(n - 1, size=hub_in_degree, replace=False).astype(np.int64)
        cand += cand >= hub  # skip the hub itself
        parts.append(hub * n + cand)
    key = np.unique(np.concatenate(parts))
    return from_edge_list(n, key % n, key // n)


def batched_small_graphs(n_graphs: int, n_min: int, n_max: int, density: float, seed: int) -> Graph:
    """Block-diagonal batch of small random graphs (batch-graph workloads).

    Graph g has n_g ~ U{n_min..n_max} nodes; every ordered pair (a != b) inside
    a graph is an edge with probability `density`; every node has a self-loop.
    """
    rng = _rng(seed, 0)
    sizes = rng.integers(n_min, n_max + 1, size=n_graphs, dtype=np.int64)
    batch_ptr = np.zeros(n_graphs + 1, dtype=np.int64)
    np.cumsum(sizes, out=batch_ptr[1:])
    srcs, dsts = [], []
    for g in range(n_graphs):
        ng = int(sizes[g])
        adj = rng.random((ng, ng)) < density
        np.fill_diagonal(adj, True)
        d, s = np.nonzero(adj)  # row-major: dst ascending, src ascending
        srcs.append(s + batch_ptr[g])
        dsts.append(d + batch_ptr[g])
    n = int(batch_ptr[-1])
    return from_edge_list(n, np.concatenate(srcs), np.concatenate(dsts), batch_ptr=batch_ptr)


def complete_graph(n: int) -> Graph:
    """Every ordered pair including self-loops: the layer reduces to dense attention."""
    d, s = np.divmod(np.arange(n * n, dtype=np.int64), n)
    return from_edge_list(n, s, d)


def tiny_graph(kind: str, seed: int = 0, n: int = 24) -> Graph:
    """Small adversarial graphs for unit tests.

    kinds: 'random'  - Erdos-Renyi-like with some empty rows and degree-1 rows;
           'hub'     - one destination connected to everyone, others sparse;
           'selfloop'- only self-loops (every row has degree 1);
           'empty'   - no edges at all;
           'dups'    - random with repeated edges kept as separate entries;
           'unsorted'- random, sources shuffled inside each row;
           'chain'   - i <- i-1 (row 0 empty).
    """
    rng = _rng(seed, 7)
    if kind == "empty":
        return from_edge_list(n, [], [])
    if kind == "selfloop":
        r = np.arange(n)
        return from_edge_list(n, r, r)
    if kind == "chain":
        r = np.arange(1, n)
        return from_edge_list(n, r - 1, r)
    m = 3 * n
    src = rng.integers(0, n, size=m)
    dst = rng.integers(0, n, size=m)
    # force a few empty rows and a few degree-1 rows
    empty_rows = np.array([1, n // 2])
    keep = ~np.isin(dst, empty_rows)
    src, dst = src[keep], dst[keep]
    single = n - 2
    keep = dst != single
    src, dst = np.append(src[keep], 3), np.append(dst[keep], single)
    if kind == "random":
        return from_edge_list(n, src, dst, dedupe=True)
    if kind == "hub":
        hub = 5
        src = np.concatenate([src, np.arange(n)])
        dst = np.concatenate([dst, np.full(n, hub)])
        return from_edge_list(n, src, dst, dedupe=True)
    if kind == "dups":
        src = np.concatenate([src, src[:n]])
        dst = np.concatenate([dst, dst[:n]])
        return from_edge_list(n, src, dst, dedupe=False)
    if kind == "unsorted":
        g = from_edge_list(n, src, dst, dedupe=True)
        idx = g.indices.copy()
        for i in range(n):
            seg = idx[g.indptr[i]:g.indptr[i + 1]]
            rng.shuffle(seg)
        return Graph(g.n, g.indptr, idx)
    raise ValueError(f"unknown tiny graph kind {kind!r}")
