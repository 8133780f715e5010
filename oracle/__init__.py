"""CPU oracle for the fused AT-GNN layer (test infrastructure only).

Nothing under this directory is imported by the product package.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may use it.
"""
from .reference import Layer, forward, backward, build_oracle  # noqa: F401
from .sched_oracle import schedule, csc_transpose  # noqa: F401
