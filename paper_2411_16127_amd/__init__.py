"""MI355X-native fused attention-GNN layer (GT / GAT / AGNN): thin Python binding over libdfgnn.so.

All computation happens in the HIP library behind the C ABI of include/dfgnn.h; this package only
marshals arguments (torch is used for device memory and streams).  There is no CPU fallback: calling
a compute entry point without the built library or without a GPU raises.
"""
from .binding import (  # noqa: F401
    DfgnnError,
    Layer,
    SchedParams,
    Graph,
    lib,
    library_path,
    status_string,
    last_error,
    version,
    graph_meta_bytes,
    graph_create,
    graph_create_batch,
    graph_destroy,
    graph_set_batch,
    graph_batch_bytes,
    graph_query,
    workspace_bytes,
    forward,
    forward_static,
    backward,
    forward_edge_bias,
    backward_edge_bias,
    attention_weights,
    probe_gather,
    timing_enable,
    timing_collect,
    QUERY,
)
