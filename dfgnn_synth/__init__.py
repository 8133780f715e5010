"""Seeded synthetic inputs (graphs and feature tensors) for the fused AT-GNN layer.

This package only manufactures inputs: CSR-by-destination graphs with the
degree structure of the evaluated workloads (dataset table of Sec. 5.1) and
random feature tensors.  It contains none of the layer's arithmetic and is
the one module that both the CPU oracle's tests and the HIP path's tests use.
"""
from .graphs import (  # noqa: F401
    Graph,
    chung_lu_graph,
    batched_small_graphs,
    hub_graph,
    complete_graph,
    tiny_graph,
    from_edge_list,
)
from .workloads import (  # noqa: F401
    WORKLOADS,
    Workload,
    make_workload,
    make_features,
    round_to_bf16,
)
