#!/usr/bin/env python3
"""Benchmark of the fused AT-GNN layer (forward + backward) on one MI355X.

One step = one forward call plus one backward call of the layer over one synthetic graph, everything
resident in HBM before the timed region.  Prints ONE JSON line:
  metric/value : fwd+bwd throughput in GEdges/s  (E / (t_fwd + t_bwd)), E = stored edges incl. self-loops
  roofline     : the kernel with the largest share of the step, its algorithmic bytes (gather model: every
                 neighbour row counted once per edge) over its mean duration from HIP events recorded on
                 the launch stream during the timed steps, against the 8 TB/s HBM peak.  This is an
                 effective rate: rows served by the Infinity Cache count like rows from HBM (the counters
                 behind `traffic` sit between L2 and the memory side and cannot tell the two apart);
                 `bare_gather` = the same rows read by a kernel that does nothing else, timed in this run
  cpu_baseline : the CPU oracle timed on a bounded sample of rows of the same graph (one thread)

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1..cfg5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "measured_traffic.md")


def measured_traffic(workload: str, kernel: str):
    """Bytes per launch between L2 and the memory side (Infinity Cache + HBM) of one pass kernel, from the
    table under profiles/ that the rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by the copy
    calibration) were summarised into.  The table records the hash of the layer-kernel sources it was measured
    on: when the sources in the tree differ, the figure is stale and None is returned."""
    from paper_2411_16127_amd.build import kernels_id
    try:
        lines = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return None
    current = kernels_id()
    for line in lines:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0] == workload and cells[1] == kernel:
            return int(cells[2]) if cells[3].strip("`") == current else None
    return None


DESCRIPTIONS = {
    "cfg1": "cfg1: GT fp32, Chung-Lu power-law graph N=2,708 (exponent 2.5) + self-loops, H=1 D=64",
    "cfg2": "cfg2: GT bf16, 1,024 disjoint graphs of 10-40 nodes, density 0.3, block-diagonal CSR, H=8 D=16",
    "cfg3": "cfg3: GAT fp32, Chung-Lu power-law graph N=169,343 (exponent 2.2) + self-loops, H=8 D=8",
    "cfg4": "cfg4: AGNN fp32, N=1,000,000 uniform edges (mean degree 8) + 16 hubs x 200,000 in-edges, H=1 D=64",
    "cfg5": "cfg5: GT fp32, Chung-Lu power-law graph N=2,449,029, ~122.5M edges (exponent 2.1) + self-loops, H=8 D=16",
}


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes(w, graph, edge_bias=False):
    """Bytes each kernel must move if no neighbour row were ever reused from cache (gather model).

    R = bytes of one node row, s = 4*H bytes of one fp32 scalar per head; per-edge and per-row figures of
    each pass.  One launch of a pass kernel covers every edge and every row (or column) of the graph.
    """
    b = 4 if w.dtype == "f32" else 2
    R, s = w.H * w.D * b, 4 * w.H
    per = {  # pass: (per edge, per node)
        "gt": {"fwd": (2 * R + 4, 2 * R + 2 * s + 4), "bwd_row": (2 * R + 4, 4 * R + 4 * s + 4),
               "bwd_col": (2 * R + 2 * s + 4, 4 * R + 4)},
        "gat": {"fwd": (R + s + 4, R + 3 * s + 4), "bwd_row": (R + s + 4, 2 * R + 6 * s + 4),
                "bwd_col": (R + 3 * s + 4, 2 * R + 3 * s + 4)},
        "agnn": {"fwd": (R + s + 4, 2 * R + 3 * s + 4), "bwd_row": (R + s + 4, 4 * R + 4 * s + 4),
                 "bwd_col": (2 * R + 3 * s + 4, 3 * R + s + 4)},
        # GATv2: one neighbour row per edge forward and in the row pass (plus the fp32 per-row share of da),
        # destination features, dO and the packed statistics per edge in the column pass
        "gatv2": {"fwd": (R + 4, 2 * R + 2 * s + 4), "bwd_row": (R + 4, 4 * R + 4 * w.H * w.D + 4 * s + 4),
                  "bwd_col": (2 * R + 2 * s + 4, 2 * R + 4)},
    }[w.model]
    if edge_bias:  # the edge term is read by every pass (the column pass also reads its position); dS is
        # written by the row pass for fp32 layers and by the column pass for bf16 layers
        f32 = w.dtype == "f32"
        extra = {"fwd": s, "bwd_row": 2 * s if f32 else s, "bwd_col": s + 4 if f32 else 2 * s + 4}
        per = {name: (pe + extra[name], pn) for name, (pe, pn) in per.items()}
    res = {name: pe * graph.nnz + pn * graph.n for name, (pe, pn) in per.items()}
    # dense-tile kernels for batches of small graphs do the work of the same passes in one launch each
    res["dense_fwd"] = res["fwd"]
    res["dense_bwd"] = res["bwd_row"] + res["bwd_col"]
    res["bwd_row_col"] = res["bwd_row"] + res["bwd_col"]  # both sides in one launch (small graphs)
    if w.model == "gt":  # two-kernel comparator: the scores make a round trip through memory
        res["fwd_scores"] = (R + s + 8) * graph.nnz + R * graph.n  # q_i counted once per row, as in the fused pass
        res["fwd_softmax_spmm"] = (R + s + 4) * graph.nnz + (R + 2 * s + 4) * graph.n
    if w.model == "gat":
        res["param_reduce"] = graph.n * (R + 2 * s)
    if w.model == "gatv2":
        res["param_reduce"] = graph.n * 4 * w.H * w.D
    if w.model == "agnn":
        res["param_reduce"] = graph.n * s
    return res


SCRUB_BYTES = 512 << 20  # twice the 256 MB Infinity Cache; written before a call to start it with cold caches


def compulsory_bytes(w, graph, edge_bias=False):
    """Bytes of one forward + backward step if every array were moved exactly once (perfect caches): the
    floor under the gather model of algorithmic_bytes.  Forward reads the input tensors and the CSR and
    writes the output and the statistics; backward reads inputs, output, upstream gradient, statistics,
    CSR and CSC and writes one gradient per input tensor."""
    b = 4 if w.dtype == "f32" else 2
    T, S = graph.n * w.H * w.D * b, graph.n * 4 * w.H
    n_in = {"gt": 3, "gat": 1, "agnn": 1, "gatv2": 2}[w.model]
    csr = 4 * (graph.n + 1) + 4 * graph.nnz
    fwd = (n_in + 1) * T + 2 * S + csr
    bwd = (2 * n_in + 2) * T + 2 * S + 2 * csr
    if edge_bias:  # read forward and backward (with its CSC positions), gradient written once
        fwd += graph.nnz * 4 * w.H
        bwd += graph.nnz * (8 * w.H + 4)
    return fwd + bwd


def sample_subproblem(graph, feats, target_edges: int, seed: int, n_cols: int = 8, max_out_degree: int = 64):
    """Random rows of the graph (whole neighbourhoods) until ~target_edges edges, relabelled compactly, plus
    a few random source nodes of small out-degree with their own row and every row they feed, so that the
    sub-problem also holds complete column-side gradients (dK, dV, or dWh / dh) for those nodes.

    The sampled rows keep their neighbour lists; nodes that only appear as neighbours become empty rows.
    Returns the sub-graph, its features, the sampled rows and the complete columns (original and new ids).
    """
    from dfgnn_synth import from_edge_list
    rng = np.random.default_rng(seed)
    deg = graph.degrees()
    order = rng.permutation(graph.n)
    take = int(np.searchsorted(np.cumsum(deg[order]), target_edges)) + 1
    rows = order[:take]
    out_deg = np.bincount(graph.indices, minlength=graph.n)
    cand = order[::-1][:4096]
    cols = np.sort(cand[(out_deg[cand] > 0) & (out_deg[cand] <= max_out_degree)][:n_cols])
    if cols.size:
        edge_pos = np.flatnonzero(np.isin(graph.indices, cols))
        feed = np.searchsorted(graph.indptr, edge_pos, side="right") - 1  # destination row of those edges
        rows = np.concatenate([rows, cols, feed])
    rows = np.unique(rows)
    starts, ends = graph.indptr[rows].astype(np.int64), graph.indptr[rows + 1].astype(np.int64)
    pos = np.concatenate([np.arange(a, b_) for a, b_ in zip(starts, ends)]) if rows.size else np.empty(0, np.int64)
    src = graph.indices[pos].astype(np.int64)
    nodes, inv = np.unique(np.concatenate([rows, src]), return_inverse=True)
    new_rows = inv[:rows.size]
    new_src = inv[rows.size:]
    new_dst = np.repeat(new_rows, (ends - starts))
    sub = from_edge_list(nodes.size, new_src, new_dst, sort=False)
    sub_feats = {k: (v[nodes] if v.ndim == 3 else v) for k, v in feats.items()}
    return sub, sub_feats, rows, new_rows, cols, np.searchsorted(nodes, cols), int(src.size)


def gather_calibration(torch, dfgnn) -> dict:
    """Rate of random row reads on this GPU, measured with the library's yardstick kernel (the gather instruction
    of the pass kernels and nothing else): what `roofline.achieved` of a gather-bound pass can reach at most."""
    gen = torch.Generator(device="cuda").manual_seed(7)
    n_idx = 1 << 26
    out = torch.empty(8192 * 64 * 4, dtype=torch.int32, device="cuda")  # 8,192 wavefronts = 32 per compute unit
    cases = []
    for row_bytes in (128, 256, 512):
        for table_mib in (64, 1024, 3072):
            n_rows = table_mib * (1 << 20) // row_bytes
            table = torch.zeros(n_rows * row_bytes // 4, dtype=torch.int32, device="cuda")
            for kind in ("uniform", "power-law"):
                if kind == "uniform":
                    idx = torch.randint(0, n_rows, (n_idx,), dtype=torch.int32, device="cuda", generator=gen)
                else:  # popularity ~ rank^-0.9 as in the power-law workloads, ranks scattered over the table
                    u = torch.rand(n_idx, device="cuda", generator=gen, dtype=torch.float64)
                    rank = ((u * (float(n_rows) ** 0.1 - 1.0) + 1.0) ** 10.0 - 1.0).clamp_(0, n_rows - 1).to(torch.int64)
                    idx = ((rank * 2654435761) % n_rows).to(torch.int32)
                for _ in range(2):
                    dfgnn.probe_gather(table, row_bytes, idx, out)
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                reps = 5
                ev[0].record()
                for _ in range(reps):
                    dfgnn.probe_gather(table, row_bytes, idx, out)
                ev[1].record()
                torch.cuda.synchronize()
                ms = ev[0].elapsed_time(ev[1]) / reps
                cases.append({"row_bytes": row_bytes, "table_MiB": table_mib, "indices": kind, "ms": round(ms, 4),
                              "GBps": round(n_idx * (row_bytes + 4) / ms / 1e6, 1)})
                del idx
            del table
    # rate against the wavefronts in flight (the size of `out` sets the launch): what the loads a kernel
    # keeps outstanding are worth; 4 KB of rows per wavefront for every row size
    sweep = []
    for row_bytes, table_mib in ((128, 122), (256, 244), (512, 1196)):
        n_rows = table_mib * (1 << 20) // row_bytes
        table = torch.zeros(n_rows * row_bytes // 4, dtype=torch.int32, device="cuda")
        idx = torch.randint(0, n_rows, (n_idx // 2,), dtype=torch.int32, device="cuda", generator=gen)
        for waves in (1024, 2048, 3072, 4096, 6144, 8192, 16384):
            small = torch.empty(waves * 64 * 4, dtype=torch.int32, device="cuda")
            for _ in range(2):
                dfgnn.probe_gather(table, row_bytes, idx, small)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record()
            for _ in range(5):
                dfgnn.probe_gather(table, row_bytes, idx, small)
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1]) / 5
            sweep.append({"row_bytes": row_bytes, "table_MiB": table_mib, "waves_per_simd": waves / 1024,
                          "GBps": round(idx.numel() * (row_bytes + 4) / ms / 1e6, 1)})
        del table, idx
    # the index arrays of the two HBM-sized workloads themselves, against one tensor of their row size
    from dfgnn_synth import make_workload
    from dfgnn_synth.workloads import make_graph
    for name in ("cfg5", "cfg4"):
        w = make_workload(name)
        graph = make_graph(w)
        row_bytes = w.H * w.D * 4
        table = torch.zeros(graph.n * row_bytes // 4, dtype=torch.int32, device="cuda")
        idx = torch.from_numpy(graph.indices).cuda()
        for _ in range(2):
            dfgnn.probe_gather(table, row_bytes, idx, out)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(5):
            dfgnn.probe_gather(table, row_bytes, idx, out)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / 5
        cases.append({"row_bytes": row_bytes, "table_MiB": round(graph.n * row_bytes / 2**20, 1), "indices": f"{name} (CSR order)",
                      "reads": int(graph.nnz), "ms": round(ms, 4), "GBps": round(graph.nnz * (row_bytes + 4) / ms / 1e6, 1)})
        del table, idx
    return {"gather_calibration": cases, "waves_in_flight_sweep": sweep, "reads": n_idx,
            "bytes_counted": "row_bytes + 4 (the index) per read"}


def cpu_baseline(w, graph, feats, target_edges: int):
    import oracle
    sub, sf, rows, new_rows, cols, new_cols, n_edges = sample_subproblem(graph, feats, target_edges, seed=w.seed + 7)
    L = oracle.Layer(w.model, w.H, w.D, scale=w.scale, neg_slope=w.neg_slope, eps=w.eps)
    kw = dict(x=sf["q"] if w.model == "gt" else sf["feat"], k=sf.get("k"), v=sf.get("v"), a_l=sf.get("a_l"),
              a_r=sf.get("a_r"))
    kw = {k: (None if v is None else np.asarray(v, dtype=np.float64)) for k, v in kw.items()}
    g64 = np.asarray(sf["d_out"], dtype=np.float64)
    oracle.build_oracle()
    # the oracle is single-threaded; its thread stays on one core while it is timed
    allowed = sorted(os.sched_getaffinity(0))
    core = allowed[len(allowed) // 2]
    os.sched_setaffinity(0, {core})
    try:
        t0 = time.perf_counter()
        fw = oracle.forward(L, sub.indptr, sub.indices, **kw)
        t1 = time.perf_counter()
        bw = oracle.backward(L, sub.indptr, sub.indices, d_out=g64, **kw)
        t2 = time.perf_counter()
    finally:
        os.sched_setaffinity(0, allowed)
    secs = t2 - t0
    info = {"value": n_edges / secs / 1e9, "unit": "GEdges/s", "cores": 1, "kind": "oracle",
            "sample": f"{rows.size} random rows with their whole neighbourhoods ({n_edges} edges) of the same graph, "
                      f"fwd {t1 - t0:.2f} s + bwd {t2 - t1:.2f} s, fp64, one thread pinned to core {core} of {os.cpu_count()} host cores"}
    return info, (rows, new_rows, cols, new_cols, fw, bw)


def sample_parity(w, timed, sample) -> dict:
    """Spot check of the buffers the timed steps left behind against the oracle's sub-problem: the output and
    the statistics of the sampled rows, the gradients that are complete inside the sub-problem (row-side ones
    of the sampled rows, every gradient of the complete columns).  Bounds as in the parity tests: fp32
    1e-5 + 1e-4 |ref|, bf16 1e-5 + 2e-2 |ref|, fp16 1e-5 + 2e-3 |ref| (2e-5 absolute for gradients of 16-bit layers)."""
    import torch
    rows, new_rows, cols, new_cols, fw, bw = sample
    rtol = {"f32": 1e-4, "bf16": 2e-2, "f16": 2e-3}[w.dtype]
    at_rows = {"out": fw["out"], "row_max": fw["row_max"], "row_sum": fw["row_sum"]}
    at_cols = {}
    if w.model in ("gt", "gatv2"):
        at_rows["d_x"] = bw["d_x"]
        at_cols["d_k"] = bw["d_k"]
        if w.model == "gt":
            at_cols["d_v"] = bw["d_v"]
    else:  # GAT, AGNN: the gradient of a node's features has a row-side and a column-side part
        at_cols["d_x"] = bw["d_x"]
    checked = {}
    for where, ids, new_ids in ((at_rows, rows, new_rows), (at_cols, cols, new_cols)):
        pick = torch.from_numpy(np.asarray(ids)).cuda()
        for name, ref_all in where.items():
            if ids.size == 0:
                continue
            got = timed[name][pick].float().cpu().numpy().astype(np.float64)
            ref = ref_all[new_ids]
            fin = np.isfinite(ref)
            atol = 2e-5 if (w.dtype != "f32" and name.startswith("d_")) else 1e-5  # 16-bit gradients: see tests/gpu_harness.py
            ok = np.array_equal(fin, np.isfinite(got)) and bool(np.all(np.abs(got[fin] - ref[fin]) <= atol + rtol * np.abs(ref[fin])))
            checked[name] = ok
    return checked


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", choices=sorted(DESCRIPTIONS))
    ap.add_argument("--super-threshold", type=int, default=0)
    ap.add_argument("--chunk-edges", type=int, default=0)
    ap.add_argument("--no-short-rows", action="store_true", help="ablation: one wavefront for every row below the super threshold")
    ap.add_argument("--no-dense-batch", action="store_true", help="ablation: general kernels also for batches of small graphs")
    ap.add_argument("--no-xcd-groups", action="store_true", help="ablation: workgroups dealt round-robin to the XCDs for every graph")
    ap.add_argument("--no-paired-passes", action="store_true", help="ablation: backward row side and column side always as separate launches")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture one step (forward + backward) into a HIP graph and replay it K times in the timed region")
    ap.add_argument("--force-dense-batch", action="store_true", help="dense-tile batch kernels whenever they apply")
    ap.add_argument("--edge-bias", action="store_true",
                    help="variant: add a seeded N(0,1) per-edge term [E,H] to the scores and compute its gradient")
    ap.add_argument("--scores-in-memory", action="store_true",
                    help="comparator: GT forward as an edge-parallel SDDMM kernel that writes the scores plus a softmax+SpMM kernel")
    ap.add_argument("--set", action="append", default=[], metavar="FIELD=VALUE",
                    help="override a field of the workload (e.g. n_graphs=2048, n_min=60, density=0.5, H=4, D=32); "
                         "the result is then a variant, named in config.workload")
    ap.add_argument("--cpu-edges", type=int, default=0, help="edges in the CPU-baseline sample (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not record per-kernel HIP events")
    ap.add_argument("--attention-weights", action="store_true",
                    help="also time the attention-weight output (normalised scores per edge from a forward call's statistics)")
    ap.add_argument("--cold", action="store_true",
                    help="cold-cache timings (512 MiB overwritten before every call) also for the workloads whose tensors "
                         "exceed the caches; they are always taken for cfg1-cfg3")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy 5 times (scale reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--gather-calibration", action="store_true",
                    help="only time the library's random-row-read yardstick (rows of 128 / 256 / 512 bytes, uniform and "
                         "power-law indices, tables inside and beyond the Infinity Cache) and print one JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2411_16127_amd as dfgnn
    from paper_2411_16127_amd import build as lib_build
    lib_build.require_current()  # load what is built; build only if nothing is; refuse a stale library
    from dfgnn_synth import make_workload, make_features
    from dfgnn_synth.workloads import make_graph

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_each_way": src.numel() * 4, "launches": 5}))
        return 0
    if args.gather_calibration:
        print(json.dumps(gather_calibration(torch, dfgnn)))
        return 0
    overrides = {}
    for item in args.set:
        key, val = item.split("=", 1)
        overrides[key] = type(getattr(make_workload(args.workload), key))(val)
    w = make_workload(args.workload, **overrides)
    t0 = time.perf_counter()
    graph = make_graph(w)
    feats = make_features(w, graph.n)
    log(f"{w.name}: N={graph.n} E={graph.nnz} generated in {time.perf_counter() - t0:.1f} s")

    sched = dfgnn.SchedParams(args.super_threshold, args.chunk_edges,
                              (1 if args.no_short_rows else 0) | (2 if args.no_dense_batch else 0) |
                              (4 if args.force_dense_batch else 0) | (8 if args.scores_in_memory else 0) |
                              (16 if args.no_xcd_groups else 0) | (64 if args.no_paired_passes else 0))
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[w.dtype]
    dev = lambda a: torch.from_numpy(a).cuda().to(tdt).contiguous()
    x = dev(feats["q"] if w.model == "gt" else feats["feat"])
    k = dev(feats["k"]) if w.model in ("gt", "gatv2") else None
    v = dev(feats["v"]) if w.model == "gt" else None
    a_l = torch.from_numpy(feats["a_l"]).cuda() if w.model in ("gat", "gatv2") else None
    a_r = torch.from_numpy(feats["a_r"]).cuda() if w.model == "gat" else None
    d_out = dev(feats["d_out"])

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g = dfgnn.Graph(graph.indptr, graph.indices, sched, batch_ptr=graph.batch_ptr)
    torch.cuda.synchronize()
    preprocess_ms = (time.perf_counter() - t0) * 1e3
    T, C = g.query("n_super_threshold"), g.query("n_chunk_edges")
    log(f"graph_create (scheduler + CSC, incl. upload): {preprocess_ms:.1f} ms; T={T} C={C}; super rows {g.query('n_super_rows')}, "
        f"super cols {g.query('n_super_cols')}")

    # the library call alone: inputs already on the device, caller's buffers allocated beforehand; median of
    # a few calls (a batch: metadata and batch structure in one call, as a training loop would make it per mini-batch)
    mb, sb = dfgnn.graph_meta_bytes(graph.n, graph.nnz, sched)
    meta2 = torch.empty(mb, dtype=torch.uint8, device="cuda")
    scratch2 = torch.empty(sb, dtype=torch.uint8, device="cuda")
    if graph.batch_ptr is not None:
        n_graphs = int(g.batch_ptr.numel() - 1)
        bb = dfgnn.graph_batch_bytes(graph.n, n_graphs)
        batch2 = torch.empty(bb, dtype=torch.uint8, device="cuda")
        create = lambda: dfgnn.graph_create_batch(graph.n, graph.nnz, g.indptr, g.indices, g.batch_ptr, n_graphs, sched,
                                                  meta2, mb, batch2, bb, scratch2, sb)
    else:
        create = lambda: dfgnn.graph_create(graph.n, graph.nnz, g.indptr, g.indices, sched, meta2, mb, scratch2, sb)
    times = []
    for _ in range(3 if graph.nnz > 50_000_000 else 11):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        h2 = create()
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3)
        dfgnn.graph_destroy(h2)
    graph_create_ms = float(np.median(times))
    del meta2, scratch2
    log(f"{'dfgnn_graph_create_batch' if graph.batch_ptr is not None else 'dfgnn_graph_create'} alone "
        f"(device-resident CSR, median of {len(times)}): {graph_create_ms:.3f} ms")

    L = dfgnn.Layer(w.model, w.H, w.D, dtype=w.dtype, scale=w.scale, neg_slope=w.neg_slope, eps=w.eps)
    N, H = graph.n, w.H
    out = torch.empty_like(x)
    row_max = torch.empty((N, H), dtype=torch.float32, device="cuda")
    row_sum = torch.empty((N, H), dtype=torch.float32, device="cuda")
    d_x = torch.empty_like(x)
    d_k = torch.empty_like(x) if w.model in ("gt", "gatv2") else None
    d_v = torch.empty_like(x) if w.model == "gt" else None
    d_a_l = torch.empty((H, w.D), dtype=torch.float32, device="cuda") if w.model in ("gat", "gatv2") else None
    d_a_r = torch.empty((H, w.D), dtype=torch.float32, device="cuda") if w.model == "gat" else None
    d_scale = torch.empty(1, dtype=torch.float32, device="cuda") if w.model == "agnn" else None
    fwd_b, bwd_b = dfgnn.workspace_bytes(g.handle, L)
    ws = torch.empty(max(fwd_b, bwd_b, 256), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    bias = d_bias = None
    if args.edge_bias:
        gen = torch.Generator(device="cuda").manual_seed(w.seed + 3)
        bias = torch.randn((graph.nnz, H), dtype=torch.float32, device="cuda", generator=gen)
        d_bias = torch.empty_like(bias)

    def fwd():
        if bias is None:
            dfgnn.forward(g.handle, L, x, k, v, a_l, a_r, out, row_max, row_sum, ws, ws.numel(), stream)
        else:
            dfgnn.forward_edge_bias(g.handle, L, x, k, v, a_l, a_r, bias, out, row_max, row_sum, ws, ws.numel(), stream)

    def bwd():
        if bias is None:
            dfgnn.backward(g.handle, L, x, k, v, a_l, a_r, out, row_max, row_sum, d_out, d_x, d_k, d_v, d_a_l, d_a_r,
                           d_scale, ws, ws.numel(), stream)
        else:
            dfgnn.backward_edge_bias(g.handle, L, x, k, v, a_l, a_r, bias, out, row_max, row_sum, d_out, d_x, d_k, d_v,
                                     d_a_l, d_a_r, d_scale, d_bias, ws, ws.numel(), stream)

    for _ in range(args.warmup):
        fwd(); bwd()
    torch.cuda.synchronize()

    # separate fwd / bwd split (not the headline number): events around each call, K iterations, median and
    # minimum.  With `scrub` a buffer twice the size of the Infinity Cache is overwritten before every call,
    # outside the events, so the call starts with none of its operands in any cache.
    scrub_buf = None

    def per_call_times(scrub: bool):
        nonlocal scrub_buf
        if scrub and scrub_buf is None:
            scrub_buf = torch.empty(SCRUB_BYTES // 4, dtype=torch.float32, device="cuda")
        rec = []
        for it in range(args.steps):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            if scrub:
                scrub_buf.fill_(float(it))
            e[0].record(stream); fwd(); e[1].record(stream)
            if scrub:
                scrub_buf.fill_(float(it) + 0.5)
            e[2].record(stream); bwd(); e[3].record(stream)
            rec.append(e)
        torch.cuda.synchronize()
        f = np.array([e[0].elapsed_time(e[1]) for e in rec])
        b = np.array([e[2].elapsed_time(e[3]) for e in rec])
        return f, b

    f_warm, b_warm = per_call_times(False)
    fwd_ms, bwd_ms = float(np.median(f_warm)), float(np.median(b_warm))

    # ---- timed region: exactly K steps between synchronisations ----
    # Per-kernel HIP events are recorded by the library on the launch stream.  Two event records per kernel
    # cost microseconds of host and queue time, which would distort steps that themselves take tens of
    # microseconds: for such workloads the events are recorded in a second pass of K steps instead.
    events_inline = (not args.no_kernel_events) and (fwd_ms + bwd_ms) >= 1.0 and not args.hip_graph
    replay = None
    if args.hip_graph:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        cg = torch.cuda.CUDAGraph()
        main_stream, stream = stream, side
        with torch.cuda.stream(side):
            fwd(); bwd()
            torch.cuda.synchronize()
            with torch.cuda.graph(cg, stream=side):
                fwd(); bwd()
        stream = main_stream
        torch.cuda.synchronize()
        replay = cg.replay
        replay()
    dfgnn.timing_enable(events_inline)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if replay:
            replay()
        else:
            fwd(); bwd()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernels = dfgnn.timing_collect() if events_inline else {}
    dfgnn.timing_enable(False)
    events_where = "timed region" if events_inline else "none"
    if not args.no_kernel_events and not events_inline:
        dfgnn.timing_enable(True)
        for _ in range(args.steps):
            fwd(); bwd()
        torch.cuda.synchronize()
        kernels = dfgnn.timing_collect()
        dfgnn.timing_enable(False)
        events_where = "separate pass of the same K steps right after the timed region"
    ms_per_step = elapsed * 1e3 / args.steps
    gedges = graph.nnz / (ms_per_step * 1e-3) / 1e9
    log(f"{ms_per_step:.3f} ms/step (fwd {fwd_ms:.3f} + bwd {bwd_ms:.3f}), {gedges:.3f} GEdges/s")

    model_bytes = algorithmic_bytes(w, graph, args.edge_bias)
    kern = {}
    for label, (ms, launches) in kernels.items():
        avg = ms / max(launches, 1)
        kb = model_bytes.get(label)
        kern[label] = {"avg_ms": round(avg, 4), "launches_per_step": launches / args.steps,
                       "algorithmic_GB": None if kb is None else round(kb / 1e9, 4),
                       "GBps": None if kb is None or avg <= 0 else round(kb / 1e9 / (avg * 1e-3), 1)}
    roofline = None
    if kern:
        dom = max(kern, key=lambda n: kern[n]["avg_ms"] * kern[n]["launches_per_step"])
        achieved = kern[dom]["GBps"]
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": None if achieved is None else round(achieved / HBM_PEAK_GBPS, 4),
                    # counters were collected for the workloads as defined, not for variants of them
                    "traffic": None if (args.set or args.edge_bias or args.scores_in_memory) else measured_traffic(w.name, dom),
                    "algorithmic_bytes_per_launch": model_bytes.get(dom), "avg_ms": kern[dom]["avg_ms"]}
    # The same rows read by a kernel that does nothing else (the library's yardstick, timed here): the
    # dominant pass walks `walk` (CSR or CSC index array) and gathers `tensors` node rows per edge.
    tensors = {"gt": {"fwd": 2, "bwd_row": 2, "bwd_col": 2, "bwd_row_col": 4}, "gat": {"fwd": 1, "bwd_row": 1, "bwd_col": 1},
               "agnn": {"fwd": 1, "bwd_row": 1, "bwd_col": 2}, "gatv2": {"fwd": 1, "bwd_row": 1, "bwd_col": 2}}[w.model]
    row_bytes = x.numel() // max(graph.n, 1) * x.element_size()
    if roofline and roofline["kernel"] in tensors and graph.n * row_bytes < (1 << 32) and row_bytes in (16, 32, 64, 128, 256, 512, 1024):
        walk = g.query("t_indices") if roofline["kernel"] == "bwd_col" else torch.from_numpy(graph.indices).cuda()
        scratch = torch.empty(8192 * 64 * 4, dtype=torch.int32, device="cuda")
        for _ in range(2):
            dfgnn.probe_gather(x, row_bytes, walk, scratch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dfgnn.probe_gather(x, row_bytes, walk, scratch)
        e1.record()
        torch.cuda.synchronize()
        bare_ms = e0.elapsed_time(e1) / 5
        n_t = tensors[roofline["kernel"]]
        roofline["bare_gather"] = {"what": "one node tensor's rows read at every entry of the index array the kernel walks, nothing else (dfgnn_probe_gather)",
                                   "ms": round(bare_ms, 4), "GBps": round(graph.nnz * (row_bytes + 4) / bare_ms / 1e6, 1),
                                   "tensors_gathered_by_kernel": n_t,
                                   "kernel_time_over_bare_reads": round(kern[roofline["kernel"]]["avg_ms"] / (n_t * bare_ms), 3)}
        del walk, scratch
    compulsory = compulsory_bytes(w, graph, args.edge_bias)
    total_model = sum(model_bytes.get(name, 0) for name in ("fwd", "bwd_row", "bwd_col", "param_reduce"))

    result = {
        "metric": "fused AT-GNN layer fwd+bwd GEdges/s at 1 GPU; achieved HBM GB/s vs peak",
        "value": round(gedges, 4), "unit": "GEdges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else f"{w.dtype} storage, f32 arithmetic", "data": "synthetic",
        "config": {"workload": DESCRIPTIONS[w.name] + (" VARIANT " + ",".join(args.set) if args.set else "") + (" + edge term" if args.edge_bias else ""), "N": graph.n, "E": graph.nnz, "H": w.H, "D": w.D,
                   "super_threshold": T, "chunk_edges": C, "xcd_group": g.query("n_xcd_group"), "stands_in_for": w.stands_in_for},
        "roofline": roofline,
        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4),
        "fwd_ms_min": round(float(f_warm.min()), 4), "bwd_ms_min": round(float(b_warm.min()), 4),
        "preprocess_ms": round(preprocess_ms, 2), "graph_create_ms": round(graph_create_ms, 4),
        # preprocessing + forward + backward as one sum, the way the end-to-end table of Sec. 5.3 adds them up
        # (per mini-batch in the batch-graph setting; value / ms_per_step above do not include preprocessing)
        "step_with_preprocess_ms": round(graph_create_ms + ms_per_step, 4),
        "step_algorithmic_GB": round(total_model / 1e9, 3),
        "step_effective_GBps": round(total_model / 1e9 / (ms_per_step * 1e-3), 1),
        "compulsory_GB": round(compulsory / 1e9, 4),
        "compulsory_time_frac": round(compulsory / (HBM_PEAK_GBPS * 1e9) / (ms_per_step * 1e-3), 4),
        "kernel_events": events_where, "launch": "hip graph replay" if args.hip_graph else "eager",
        "kernels": kern,
    }

    if args.attention_weights:
        p_out = torch.empty((graph.nnz, H), dtype=torch.float32, device="cuda")
        att = lambda: dfgnn.attention_weights(g.handle, L, x, k, a_l, a_r, bias, row_max, row_sum, p_out, stream)
        att()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            att()
        e1.record(stream)
        torch.cuda.synchronize()
        att_ms = e0.elapsed_time(e1) / args.steps
        # the neighbour row the score needs (GT: K_j without V_j; the other models score and aggregate the same
        # row), the index and the stored weight; per row the destination features, the two statistics and the
        # row pointer
        b_el = 4 if w.dtype == "f32" else 2
        R, s_ = w.H * w.D * b_el, 4 * w.H
        per_edge = {"gt": R + 4, "gat": R + 4, "agnn": R + s_ + 4, "gatv2": R + 4}[w.model] + s_ + (s_ if bias is not None else 0)
        att_bytes = per_edge * graph.nnz + (R + 2 * s_ + 4) * graph.n
        result["attention_weights"] = {"avg_ms": round(att_ms, 4), "algorithmic_GB": round(att_bytes / 1e9, 4),
                                       "GBps": round(att_bytes / 1e9 / (att_ms * 1e-3), 1),
                                       "GEdges_per_s": round(graph.nnz / (att_ms * 1e-3) / 1e9, 3)}
        del p_out
    if args.cold or w.name in ("cfg1", "cfg2", "cfg3"):
        f_cold, b_cold = per_call_times(True)
        cold_ms = float(np.median(f_cold) + np.median(b_cold))
        result["cold_cache"] = {
            "scrub_bytes_before_every_call": SCRUB_BYTES,
            "fwd_ms": round(float(np.median(f_cold)), 4), "fwd_ms_min": round(float(f_cold.min()), 4),
            "bwd_ms": round(float(np.median(b_cold)), 4), "bwd_ms_min": round(float(b_cold.min()), 4),
            "GEdges_per_s": round(graph.nnz / (cold_ms * 1e-3) / 1e9, 4),
            "compulsory_time_frac": round(compulsory / (HBM_PEAK_GBPS * 1e9) / (cold_ms * 1e-3), 4)}
        log(f"cold caches: fwd {np.median(f_cold):.3f} + bwd {np.median(b_cold):.3f} ms (warm {fwd_ms:.3f} + {bwd_ms:.3f})")
    if not args.no_cpu_baseline and not args.edge_bias:
        target = args.cpu_edges or {"cfg1": 1 << 30, "cfg2": 1 << 30, "cfg3": 1 << 30, "cfg4": 8000000, "cfg5": 10000000}[w.name]
        info, sample = cpu_baseline(w, graph, feats, target)
        # the sample doubles as a parity spot check of the buffers that were just timed (output, statistics, gradients)
        checked = sample_parity(w, {"out": out, "row_max": row_max, "row_sum": row_sum, "d_x": d_x, "d_k": d_k, "d_v": d_v}, sample)
        info["sample_parity"] = checked
        info["sample_parity_ok"] = bool(checked) and all(checked.values())
        info["gpu_over_cpu"] = round(gedges / info["value"], 1)
        info["value"] = float(f"{info['value']:.6g}")
        result["cpu_baseline"] = info
        log(f"oracle: {info['value']:.5f} GEdges/s on 1 core; sample parity ok = {info['sample_parity_ok']}")
    print(json.dumps(result), flush=True)
    g.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
