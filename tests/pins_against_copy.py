"""Runs the oracle pins against a COPY of the oracle (a library built from a changed copy of atgnn_oracle.c, or a
changed copy of sched_oracle.py).  tests/test_oracle_mutants.py starts this file as a child process; the copy is
put in place here, on the test side, for this one process: the oracle package itself has no switch that could
swap the checker, so no other run (GPU parity, smoke, benchmark) can end up checking against a copy.

    python tests/pins_against_copy.py layer <library.so>
    python tests/pins_against_copy.py sched <sched_oracle_copy.py>

Exit status: that of pytest on the pin file (0 = every pin passed)."""
import ctypes
import importlib.util
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))


def main(kind: str, path: str) -> int:
    import pytest
    import oracle
    import oracle.reference as reference
    if kind == "layer":
        lib = ctypes.CDLL(path)
        lib.atgnn_oracle_forward.restype = ctypes.c_int
        lib.atgnn_oracle_backward.restype = ctypes.c_int
        reference._lib = lib  # the handle oracle.forward / oracle.backward call through
        pins = "test_oracle_pins.py"
    elif kind == "sched":
        spec = importlib.util.spec_from_file_location("sched_oracle_copy", path)
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        oracle.schedule, oracle.csc_transpose = mod.schedule, mod.csc_transpose
        pins = "test_sched_oracle.py"
    else:
        raise SystemExit(f"unknown kind {kind!r}")
    return int(pytest.main([os.path.join(ROOT, "tests", pins), "-x", "-q", "-p", "no:cacheprovider"]))


if __name__ == "__main__":
    sys.exit(main(sys.argv[1], sys.argv[2]))
