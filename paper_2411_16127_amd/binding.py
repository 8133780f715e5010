"""ctypes binding of include/dfgnn.h.  Function names and argument order follow the C ABI.

The low-level functions (graph_meta_bytes, graph_create, graph_query, workspace_bytes, forward,
backward) take torch tensors or raw pointers and only marshal them.  `Graph` and the `alloc=True`
conveniences allocate the caller-owned buffers with torch and pass them through unchanged.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdfgnn.so")

MODEL = {"gt": 0, "gat": 1, "agnn": 2, "gatv2": 3}
DTYPE = {"f32": 0, "bf16": 1, "f16": 2}
QUERY = {
    "row_order": 0, "row_chunk_ptr": 1, "row_chunks": 2, "t_indptr": 3, "t_indices": 4, "t_eid": 5,
    "col_order": 6, "col_chunk_ptr": 7, "col_chunks": 8, "n_super_rows": 9, "n_super_cols": 10,
    "n_super_threshold": 11, "n_chunk_edges": 12, "n_batch_dense": 13, "n_xcd_group": 14,
}


class DfgnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} - {last_error()}")


class _CSched(ctypes.Structure):
    _fields_ = [("super_threshold", ctypes.c_int32), ("chunk_edges", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 5)]


class _CLayer(ctypes.Structure):
    _fields_ = [("model", ctypes.c_int32), ("dtype", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
                ("scale", ctypes.c_float), ("neg_slope", ctypes.c_float), ("eps", ctypes.c_float),
                ("reserved", ctypes.c_int32 * 1)]


@dataclass
class SchedParams:
    super_threshold: int = 0  # 0 = library default
    chunk_edges: int = 0
    flags: int = 0            # bits: 1 = no short-row mapping, 2 = no dense-tile batch kernels, 4 = dense-tile kernels whenever they apply, 8 = GT forward with scores through memory (comparator), 16 = no XCD-local runs of the work list, 32 = forward-only graph (no CSC; backward calls are refused), 64 = backward row side and column side always as separate launches

    def _c(self) -> _CSched:
        return _CSched(self.super_threshold, self.chunk_edges, self.flags, (ctypes.c_int32 * 5)())


@dataclass
class Layer:
    model: str          # 'gt' | 'gat' | 'agnn' | 'gatv2'
    H: int
    D: int
    dtype: str = "f32"  # 'f32' | 'bf16' | 'f16' (storage type of node tensors; arithmetic is fp32)
    scale: float = 1.0  # GT: score scale; AGNN: beta
    neg_slope: float = 0.2
    eps: float = 1e-12

    def _c(self) -> _CLayer:
        return _CLayer(MODEL[self.model], DTYPE[self.dtype], self.H, self.D, self.scale, self.neg_slope, self.eps,
                       (ctypes.c_int32 * 1)())


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Load libdfgnn.so (built in-tree by paper_2411_16127_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is not built: run `python -m paper_2411_16127_amd.build` "
                               "(there is no fallback implementation)")
        import torch  # noqa: F401  (first, so that the process uses the HIP runtime torch ships: device memory and streams come from it)
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
        L.dfgnn_status_string.restype = ctypes.c_char_p
        L.dfgnn_status_string.argtypes = [ctypes.c_int]
        L.dfgnn_last_error.restype = ctypes.c_char_p
        L.dfgnn_last_error.argtypes = []
        L.dfgnn_version.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.dfgnn_graph_meta_bytes.argtypes = [i64, i64, vp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.dfgnn_graph_create.argtypes = [ctypes.POINTER(vp), i64, i64, vp, vp, vp, vp, sz, vp, sz, vp]
        L.dfgnn_graph_create_batch.argtypes = [ctypes.POINTER(vp), i64, i64, vp, vp, vp, i64, vp, vp, sz, vp, sz, vp, sz, vp]
        L.dfgnn_graph_destroy.argtypes = [vp]
        L.dfgnn_graph_set_batch.argtypes = [vp, vp, i64, vp, sz, vp]
        L.dfgnn_graph_batch_bytes.argtypes = [i64, i64, ctypes.POINTER(sz)]
        L.dfgnn_graph_query.argtypes = [vp, ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(i64)]
        L.dfgnn_workspace_bytes.argtypes = [vp, vp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.dfgnn_forward.argtypes = [vp, vp] + [vp] * 8 + [vp, sz, vp]
        L.dfgnn_forward_static.argtypes = [vp, vp] + [vp] * 8 + [vp]
        L.dfgnn_backward.argtypes = [vp, vp] + [vp] * 15 + [vp, sz, vp]
        L.dfgnn_forward_edge_bias.argtypes = [vp, vp] + [vp] * 9 + [vp, sz, vp]
        L.dfgnn_attention_weights.argtypes = [vp, vp] + [vp] * 8 + [vp]
        L.dfgnn_backward_edge_bias.argtypes = [vp, vp] + [vp] * 17 + [vp, sz, vp]
        L.dfgnn_probe_gather.argtypes = [vp, i64, ctypes.c_int32, vp, i64, vp, sz, vp]
        L.dfgnn_timing_enable.argtypes = [ctypes.c_int]
        L.dfgnn_timing_collect.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int)]
        for name in ("dfgnn_graph_create_batch", "dfgnn_graph_set_batch", "dfgnn_graph_batch_bytes", "dfgnn_timing_enable", "dfgnn_timing_collect", "dfgnn_version", "dfgnn_graph_meta_bytes", "dfgnn_graph_create", "dfgnn_graph_destroy",
                     "dfgnn_graph_query", "dfgnn_workspace_bytes", "dfgnn_forward", "dfgnn_backward", "dfgnn_forward_static",
                     "dfgnn_forward_edge_bias", "dfgnn_backward_edge_bias", "dfgnn_attention_weights", "dfgnn_probe_gather"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().dfgnn_status_string(int(status)).decode()


def last_error() -> str:
    return lib().dfgnn_last_error().decode()


def version() -> Tuple[int, int]:
    a, b = ctypes.c_int(), ctypes.c_int()
    lib().dfgnn_version(ctypes.byref(a), ctypes.byref(b))
    return a.value, b.value


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise DfgnnError(rc, where)


def dtype_name(torch_dtype) -> str:
    """Layer dtype string of a torch dtype (float32 / bfloat16 / float16)."""
    import torch
    try:
        return {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}[torch_dtype]
    except KeyError:
        raise ValueError(f"node tensors must be float32, bfloat16 or float16, not {torch_dtype}") from None


def _ptr(t) -> ctypes.c_void_p:
    """Device pointer of a torch tensor (or None / int passed through)."""
    if t is None:
        return ctypes.c_void_p(None)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_cuda:
        raise ValueError("dfgnn entry points take device tensors")
    if not t.is_contiguous():
        raise ValueError("dfgnn entry points take contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def graph_meta_bytes(N: int, E: int, sched: Optional[SchedParams] = None) -> Tuple[int, int]:
    meta, scratch = ctypes.c_size_t(), ctypes.c_size_t()
    cs = sched._c() if sched else None
    _check(lib().dfgnn_graph_meta_bytes(N, E, ctypes.byref(cs) if cs else None, ctypes.byref(meta),
                                        ctypes.byref(scratch)), "dfgnn_graph_meta_bytes")
    return meta.value, scratch.value


def graph_create(N: int, E: int, d_indptr, d_indices, sched: Optional[SchedParams], d_meta, meta_bytes: int,
                 d_scratch, scratch_bytes: int, stream=None) -> ctypes.c_void_p:
    handle = ctypes.c_void_p()
    cs = sched._c() if sched else None
    _check(lib().dfgnn_graph_create(ctypes.byref(handle), N, E, _ptr(d_indptr), _ptr(d_indices),
                                    ctypes.byref(cs) if cs else None, _ptr(d_meta), meta_bytes, _ptr(d_scratch),
                                    scratch_bytes, _stream(stream)), "dfgnn_graph_create")
    return handle


def graph_create_batch(N: int, E: int, d_indptr, d_indices, d_batch_ptr, n_graphs: int, sched: Optional[SchedParams],
                       d_meta, meta_bytes: int, d_batch, batch_bytes: int, d_scratch, scratch_bytes: int,
                       stream=None) -> ctypes.c_void_p:
    handle = ctypes.c_void_p()
    cs = sched._c() if sched else None
    _check(lib().dfgnn_graph_create_batch(ctypes.byref(handle), N, E, _ptr(d_indptr), _ptr(d_indices), _ptr(d_batch_ptr),
                                          n_graphs, ctypes.byref(cs) if cs else None, _ptr(d_meta), meta_bytes,
                                          _ptr(d_batch), batch_bytes, _ptr(d_scratch), scratch_bytes, _stream(stream)),
           "dfgnn_graph_create_batch")
    return handle


def graph_batch_bytes(N: int, n_graphs: int) -> int:
    b = ctypes.c_size_t()
    _check(lib().dfgnn_graph_batch_bytes(N, n_graphs, ctypes.byref(b)), "dfgnn_graph_batch_bytes")
    return b.value


def graph_set_batch(handle, d_batch_ptr, n_graphs: int, d_batch, batch_bytes: int, stream=None) -> None:
    _check(lib().dfgnn_graph_set_batch(handle, _ptr(d_batch_ptr), n_graphs, _ptr(d_batch), batch_bytes,
                                       _stream(stream)), "dfgnn_graph_set_batch")


def graph_destroy(handle) -> None:
    _check(lib().dfgnn_graph_destroy(handle), "dfgnn_graph_destroy")


def graph_query(handle, what) -> Tuple[int, int]:
    """(device pointer, element count) of one metadata array."""
    p, c = ctypes.c_void_p(), ctypes.c_int64()
    item = QUERY[what] if isinstance(what, str) else int(what)
    _check(lib().dfgnn_graph_query(handle, item, ctypes.byref(p), ctypes.byref(c)), "dfgnn_graph_query")
    return (p.value or 0), c.value


def workspace_bytes(handle, layer: Layer) -> Tuple[int, int]:
    f, b = ctypes.c_size_t(), ctypes.c_size_t()
    cl = layer._c()
    _check(lib().dfgnn_workspace_bytes(handle, ctypes.byref(cl), ctypes.byref(f), ctypes.byref(b)),
           "dfgnn_workspace_bytes")
    return f.value, b.value


def forward(handle, layer: Layer, x, k, v, a_l, a_r, out, row_max, row_sum, workspace, workspace_bytes_: int,
            stream=None) -> None:
    cl = layer._c()
    _check(lib().dfgnn_forward(handle, ctypes.byref(cl), _ptr(x), _ptr(k), _ptr(v), _ptr(a_l), _ptr(a_r), _ptr(out),
                               _ptr(row_max), _ptr(row_sum), _ptr(workspace), workspace_bytes_, _stream(stream)),
           "dfgnn_forward")


def forward_static(handle, layer: Layer, x, k, v, a_l, a_r, out, row_max, row_sum, stream=None) -> None:
    """dfgnn_forward with the library's static scratch in place of a caller workspace (allocates nothing)."""
    cl = layer._c()
    _check(lib().dfgnn_forward_static(handle, ctypes.byref(cl), _ptr(x), _ptr(k), _ptr(v), _ptr(a_l), _ptr(a_r),
                                      _ptr(out), _ptr(row_max), _ptr(row_sum), _stream(stream)), "dfgnn_forward_static")


def backward(handle, layer: Layer, x, k, v, a_l, a_r, out, row_max, row_sum, d_out, d_x, d_k, d_v, d_a_l, d_a_r,
             d_scale, workspace, workspace_bytes_: int, stream=None) -> None:
    cl = layer._c()
    _check(lib().dfgnn_backward(handle, ctypes.byref(cl), _ptr(x), _ptr(k), _ptr(v), _ptr(a_l), _ptr(a_r), _ptr(out),
                                _ptr(row_max), _ptr(row_sum), _ptr(d_out), _ptr(d_x), _ptr(d_k), _ptr(d_v),
                                _ptr(d_a_l), _ptr(d_a_r), _ptr(d_scale), _ptr(workspace), workspace_bytes_,
                                _stream(stream)), "dfgnn_backward")


def forward_edge_bias(handle, layer: Layer, x, k, v, a_l, a_r, edge_bias, out, row_max, row_sum, workspace,
                      workspace_bytes_: int, stream=None) -> None:
    cl = layer._c()
    _check(lib().dfgnn_forward_edge_bias(handle, ctypes.byref(cl), _ptr(x), _ptr(k), _ptr(v), _ptr(a_l), _ptr(a_r),
                                         _ptr(edge_bias), _ptr(out), _ptr(row_max), _ptr(row_sum), _ptr(workspace),
                                         workspace_bytes_, _stream(stream)), "dfgnn_forward_edge_bias")


def backward_edge_bias(handle, layer: Layer, x, k, v, a_l, a_r, edge_bias, out, row_max, row_sum, d_out, d_x, d_k, d_v,
                       d_a_l, d_a_r, d_scale, d_edge_bias, workspace, workspace_bytes_: int, stream=None) -> None:
    cl = layer._c()
    _check(lib().dfgnn_backward_edge_bias(handle, ctypes.byref(cl), _ptr(x), _ptr(k), _ptr(v), _ptr(a_l), _ptr(a_r),
                                          _ptr(edge_bias), _ptr(out), _ptr(row_max), _ptr(row_sum), _ptr(d_out),
                                          _ptr(d_x), _ptr(d_k), _ptr(d_v), _ptr(d_a_l), _ptr(d_a_r), _ptr(d_scale),
                                          _ptr(d_edge_bias), _ptr(workspace), workspace_bytes_, _stream(stream)),
           "dfgnn_backward_edge_bias")


def probe_gather(table, row_bytes: int, idx, out, stream=None) -> None:
    """Measurement yardstick: read rows idx[e] (row_bytes each) of `table` and nothing else; `out` (a device
    buffer of a multiple of 4096 bytes) sets the size of the launch and receives the XOR of what each thread read."""
    n_rows = table.numel() * table.element_size() // int(row_bytes)
    _check(lib().dfgnn_probe_gather(_ptr(table), n_rows, int(row_bytes), _ptr(idx), idx.numel(), _ptr(out),
                                    out.numel() * out.element_size(), _stream(stream)), "dfgnn_probe_gather")


def attention_weights(handle, layer: Layer, x, k, a_l, a_r, edge_bias, row_max, row_sum, p, stream=None) -> None:
    cl = layer._c()
    _check(lib().dfgnn_attention_weights(handle, ctypes.byref(cl), _ptr(x), _ptr(k), _ptr(a_l), _ptr(a_r),
                                         _ptr(edge_bias), _ptr(row_max), _ptr(row_sum), _ptr(p), _stream(stream)),
           "dfgnn_attention_weights")


def timing_enable(enable: bool) -> None:
    _check(lib().dfgnn_timing_enable(1 if enable else 0), "dfgnn_timing_enable")


def timing_collect(max_labels: int = 64) -> Dict[str, Tuple[float, int]]:
    """{kernel label: (total milliseconds, launches)} since the last collect / enable."""
    labels = (ctypes.c_char_p * max_labels)()
    ms = (ctypes.c_double * max_labels)()
    launches = (ctypes.c_int64 * max_labels)()
    n = ctypes.c_int()
    _check(lib().dfgnn_timing_collect(max_labels, labels, ms, launches, ctypes.byref(n)), "dfgnn_timing_collect")
    return {labels[i].decode(): (ms[i], launches[i]) for i in range(n.value)}


class Graph:
    """Owns the device buffers of one graph (CSR arrays, metadata) and its library handle."""

    def __init__(self, indptr, indices, sched: Optional[SchedParams] = None, device="cuda:0", stream=None,
                 batch_ptr=None):
        import torch
        self.device = torch.device(device)
        self.indptr = torch.as_tensor(indptr, dtype=torch.int32).to(self.device).contiguous()
        self.indices = torch.as_tensor(indices, dtype=torch.int32).to(self.device).contiguous()
        self.N = int(self.indptr.numel() - 1)
        self.E = int(self.indices.numel())
        self.sched = sched
        meta_b, scratch_b = graph_meta_bytes(self.N, self.E, sched)
        self.meta = torch.empty(meta_b, dtype=torch.uint8, device=self.device)
        scratch = torch.empty(scratch_b, dtype=torch.uint8, device=self.device)
        self.batch_ptr = None
        if batch_ptr is None:
            self.handle = graph_create(self.N, self.E, self.indptr, self.indices, sched, self.meta, meta_b, scratch,
                                       scratch_b, stream)
        else:  # metadata and batch structure in one call
            self.batch_ptr = torch.as_tensor(batch_ptr, dtype=torch.int32).to(self.device).contiguous()
            n_graphs = int(self.batch_ptr.numel() - 1)
            nbytes = graph_batch_bytes(self.N, n_graphs)
            self.batch_meta = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.handle = graph_create_batch(self.N, self.E, self.indptr, self.indices, self.batch_ptr, n_graphs, sched,
                                             self.meta, meta_b, self.batch_meta, nbytes, scratch, scratch_b, stream)
        del scratch
        self._ws: Dict[tuple, object] = {}

    @classmethod
    def from_edge_index(cls, src, dst, num_nodes: int, sched: Optional[SchedParams] = None, device="cuda:0",
                        stream=None, batch_ptr=None):
        """Graph from an unsorted edge list (edge e goes from src[e] to dst[e]; any integer dtype, host or
        device).  Edges are grouped by destination with a stable sort, so the sources of a row keep their
        order in the list.  Returns (graph, perm): perm[t] is the list position of the edge stored at CSR
        position t, i.e. per-edge data in list order becomes CSR order by `data[perm]` (edge terms), and CSR
        order goes back with `out[perm] = data_csr`.  batch_ptr (optional, [n_graphs + 1]) announces a
        block-diagonal batch of small graphs."""
        import torch
        dev = torch.device(device)
        src = torch.as_tensor(src).to(dev).flatten().long()
        dst = torch.as_tensor(dst).to(dev).flatten().long()
        if src.numel() != dst.numel():
            raise ValueError("src and dst differ in length")
        if src.numel() and (int(src.min()) < 0 or int(dst.min()) < 0 or int(src.max()) >= num_nodes
                            or int(dst.max()) >= num_nodes):
            raise ValueError("edge endpoint out of range")
        order = torch.sort(dst, stable=True).indices
        counts = torch.bincount(dst, minlength=num_nodes)
        indptr = torch.zeros(num_nodes + 1, dtype=torch.int64, device=dev)
        indptr[1:] = torch.cumsum(counts, 0)
        return cls(indptr.to(torch.int32), src[order].to(torch.int32), sched, device, stream,
                   batch_ptr=batch_ptr), order

    @classmethod
    def from_graph_list(cls, graphs, sched: Optional[SchedParams] = None, device="cuda:0", stream=None):
        """One block-diagonal graph from a mini-batch of small graphs (the batch-graph setting of Sec. 5.1).
        graphs: sequence of (src, dst, num_nodes) with node ids local to each graph.  Returns
        (graph, perm, batch_ptr): graph b owns nodes batch_ptr[b] .. batch_ptr[b+1]-1 of the batch (node
        tensors of the graphs concatenated in order), perm as in from_edge_index over the concatenated edge
        lists.  The batch structure is announced to the library (dfgnn_graph_set_batch)."""
        import torch
        dev = torch.device(device)
        sizes = torch.tensor([int(n) for _, _, n in graphs], dtype=torch.int64)
        if sizes.numel() == 0 or int(sizes.min()) < 0:
            raise ValueError("a batch needs at least one graph, and node counts cannot be negative")
        batch_ptr = torch.zeros(sizes.numel() + 1, dtype=torch.int64)
        batch_ptr[1:] = torch.cumsum(sizes, 0)
        srcs, dsts = [], []
        for b, (src, dst, n) in enumerate(graphs):
            src = torch.as_tensor(src).to(dev).flatten().long()
            dst = torch.as_tensor(dst).to(dev).flatten().long()
            if src.numel() != dst.numel():
                raise ValueError(f"graph {b}: src and dst differ in length")
            if src.numel() and (int(src.min()) < 0 or int(dst.min()) < 0 or int(src.max()) >= n or int(dst.max()) >= n):
                raise ValueError(f"graph {b}: edge endpoint out of range")
            srcs.append(src + int(batch_ptr[b]))
            dsts.append(dst + int(batch_ptr[b]))
        bp = batch_ptr.to(torch.int32).to(dev)
        g, perm = cls.from_edge_index(torch.cat(srcs), torch.cat(dsts), int(batch_ptr[-1]), sched, device, stream,
                                      batch_ptr=bp)
        return g, perm, bp

    def close(self) -> None:
        if getattr(self, "handle", None) is not None:
            graph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def query(self, what: str):
        """Copy of one metadata array as an int32 torch tensor (counts come back as int)."""
        import torch
        p, c = graph_query(self.handle, what)
        if what.startswith("n_"):
            return c
        if c == 0:
            return torch.empty(0, dtype=torch.int32, device=self.device)
        off = p - self.meta.data_ptr()
        return self.meta[off:off + 4 * c].view(torch.int32).clone()

    def workspace(self, layer: Layer, backward_: bool):
        import torch
        f, b = workspace_bytes(self.handle, layer)
        need = b if backward_ else f
        key = (layer.model, layer.dtype, layer.H, layer.D, backward_)
        ws = self._ws.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
            self._ws[key] = ws
        return ws, need

    def _check_tensors(self, layer: Layer, node_tensors, head_tensors=(), stat_tensors=()) -> None:
        """Host-side shape / dtype checks: the C ABI carries no tensor sizes, so a wrong one would fault."""
        import torch
        want = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[layer.dtype]
        for t in node_tensors:
            if t is None:
                continue
            if t.dtype != want or t.numel() != self.N * layer.H * layer.D or t.device != self.device:
                raise ValueError(f"node tensor must be {want} with {self.N}x{layer.H}x{layer.D} elements on {self.device}")
        for t in head_tensors:
            if layer.model == "agnn":  # a_l carries beta: one float32 value on the device
                if t is not None and (t.dtype != torch.float32 or t.numel() != 1 or t.device != self.device):
                    raise ValueError(f"AGNN: a_l must be one float32 value on {self.device} (beta)")
            elif t is not None and (t.dtype != torch.float32 or t.numel() != layer.H * layer.D):
                raise ValueError("attention vectors must be float32 [H, D]")
        for t in stat_tensors:
            if t is not None and (t.dtype != torch.float32 or t.numel() != self.N * layer.H):
                raise ValueError("softmax statistics must be float32 [N, H]")

    def _check_edge_tensor(self, layer: Layer, t) -> None:
        import torch
        if t is not None and (t.dtype != torch.float32 or t.numel() != self.E * layer.H or t.device != self.device
                              or not t.is_contiguous()):
            raise ValueError(f"edge term must be contiguous float32 with {self.E}x{layer.H} elements on {self.device}")

    def forward(self, layer: Layer, x, k=None, v=None, a_l=None, a_r=None, stream=None, edge_bias=None):
        """Allocates out / row_max / row_sum and calls dfgnn_forward (dfgnn_forward_edge_bias with an edge term)."""
        import torch
        self._check_tensors(layer, (x, k, v), (a_l, a_r))
        self._check_edge_tensor(layer, edge_bias)
        out = torch.empty_like(x)
        row_max = torch.empty((self.N, layer.H), dtype=torch.float32, device=self.device)
        row_sum = torch.empty((self.N, layer.H), dtype=torch.float32, device=self.device)
        ws, need = self.workspace(layer, False)
        if edge_bias is None:
            forward(self.handle, layer, x, k, v, a_l, a_r, out, row_max, row_sum, ws, ws.numel(), stream)
        else:
            forward_edge_bias(self.handle, layer, x, k, v, a_l, a_r, edge_bias, out, row_max, row_sum, ws, ws.numel(),
                              stream)
        return out, row_max, row_sum

    def attention(self, layer: Layer, x, k, a_l, a_r, row_max, row_sum, stream=None, edge_bias=None):
        """Attention weights [E, H] (fp32, CSR edge order) from the statistics of a forward call."""
        import torch
        self._check_tensors(layer, (x, k), (a_l, a_r), (row_max, row_sum))
        self._check_edge_tensor(layer, edge_bias)
        p = torch.empty((self.E, layer.H), dtype=torch.float32, device=self.device)
        attention_weights(self.handle, layer, x, k, a_l, a_r, edge_bias, row_max, row_sum, p, stream)
        return p

    def backward(self, layer: Layer, x, k, v, a_l, a_r, out, row_max, row_sum, d_out, stream=None, edge_bias=None,
                 want_d_edge_bias: bool = True):
        """Allocates the gradient tensors and calls dfgnn_backward (dfgnn_backward_edge_bias with an edge term,
        which adds 'd_edge_bias' [E, H] to the result unless want_d_edge_bias is False); returns a dict."""
        import torch
        self._check_tensors(layer, (x, k, v, out, d_out), (a_l, a_r), (row_max, row_sum))
        self._check_edge_tensor(layer, edge_bias)
        res = {"d_x": torch.empty_like(x)}
        d_k = d_v = d_a_l = d_a_r = d_scale = None
        if layer.model == "gt":
            d_k = res["d_k"] = torch.empty_like(x)
            d_v = res["d_v"] = torch.empty_like(x)
        elif layer.model == "gat":
            d_a_l = res["d_a_l"] = torch.empty((layer.H, layer.D), dtype=torch.float32, device=self.device)
            d_a_r = res["d_a_r"] = torch.empty((layer.H, layer.D), dtype=torch.float32, device=self.device)
        elif layer.model == "gatv2":
            d_k = res["d_k"] = torch.empty_like(x)
            d_a_l = res["d_a_l"] = torch.empty((layer.H, layer.D), dtype=torch.float32, device=self.device)
        else:
            d_scale = res["d_scale"] = torch.empty(1, dtype=torch.float32, device=self.device)
        ws, need = self.workspace(layer, True)
        if edge_bias is None:
            backward(self.handle, layer, x, k, v, a_l, a_r, out, row_max, row_sum, d_out, res["d_x"], d_k, d_v, d_a_l,
                     d_a_r, d_scale, ws, ws.numel(), stream)
        else:
            d_b = None
            if want_d_edge_bias:
                d_b = res["d_edge_bias"] = torch.empty((self.E, layer.H), dtype=torch.float32, device=self.device)
            backward_edge_bias(self.handle, layer, x, k, v, a_l, a_r, edge_bias, out, row_max, row_sum, d_out,
                               res["d_x"], d_k, d_v, d_a_l, d_a_r, d_scale, d_b, ws, ws.numel(), stream)
        return res
