"""CPU oracle for the fused AT-GNN layer (test infrastructure only).

Nothing under this directory is imported by the product package.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may use it.
"""
from .reference import Layer, forward, backward, build_oracle  # noqa: F401
import os as _os

if _os.environ.get("DFGNN_SCHED_ORACLE_FILE"):
    # a copy of sched_oracle.py with a planted mistake (tests/test_oracle_mutants.py expects its pins to fail)
    import importlib.util as _ilu
    _spec = _ilu.spec_from_file_location("oracle._sched_oracle_copy", _os.environ["DFGNN_SCHED_ORACLE_FILE"])
    _mod = _ilu.module_from_spec(_spec)
    _spec.loader.exec_module(_mod)
    schedule, csc_transpose = _mod.schedule, _mod.csc_transpose
else:
    from .sched_oracle import schedule, csc_transpose  # noqa: F401
