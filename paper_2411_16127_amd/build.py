"""Builds libdfgnn.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2411_16127_amd.build [-v] [--incremental]`.

The library carries the hash of the sources it was built from (dfgnn_build_id); `stale()` compares it with the
sources in the tree, so that tests and the benchmark refuse a library that is older than an edit."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
HEADER = os.path.join(os.path.dirname(HERE), "include", "dfgnn.h")
LIB = os.path.join(HERE, "libdfgnn.so")
# the layer kernels are instantiated in one unit per model and direction so that they compile in parallel;
# the slowest units come first
SOURCES = ["layer_gt_bwd.hip", "layer_gatv2_bwd.hip", "layer_agnn_bwd.hip", "layer_gat_bwd.hip", "layer_gt_fwd.hip",
           "layer_gatv2_fwd.hip", "layer_agnn_fwd.hip", "layer_gat_fwd.hip", "dense_batch_f32.hip", "dense_batch_bf16.hip", "dense_batch.hip",
           "graph.hip", "layer.hip", "api.cpp"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed fp32 arithmetic is kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def lib_path() -> str:
    return LIB


def _digest(paths, extra: str = "") -> str:
    h = hashlib.sha256(extra.encode())
    for path in paths:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:24]


def _headers():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))) + [HEADER]


def source_id() -> str:
    """Hash of every source file, the public header and the compiler flags."""
    return _digest(sorted(os.path.join(CSRC, s) for s in SOURCES) + _headers(), " ".join(FLAGS))


def kernels_id() -> str:
    """Hash of the sources of the layer kernels alone (what the traffic counters under profiles/ were measured on)."""
    names = sorted(f for f in os.listdir(CSRC) if f.startswith(("layer", "pass_")))
    return _digest([os.path.join(CSRC, f) for f in names], " ".join(FLAGS))


def built_id() -> str:
    """The hash the library in the tree carries ('' if there is no library or it has no id).  Read from the
    file, not through dlopen: loading the library pulls in a HIP runtime, and a test process must get that
    from torch first (two HIP runtimes in one process do not see the GPU)."""
    if not os.path.exists(LIB):
        return ""
    tag = b"DFGNN_BUILD_ID="
    with open(LIB, "rb") as f:
        data = f.read()
    at = data.find(tag)
    if at < 0:
        return ""
    end = data.find(b"\0", at)
    return data[at + len(tag):end].decode(errors="replace")


def stale() -> bool:
    """True when a library exists but was built from other sources than the tree holds."""
    return os.path.exists(LIB) and built_id() != source_id()


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compile every source to an object (in parallel) and link the shared library.  With `incremental`, an
    object whose source, headers and flags are unchanged since it was compiled is kept."""
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()
    build_id = source_id()
    headers = _headers()

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        stamp = obj + ".id"
        flags = FLAGS + ([f'-DDFGNN_BUILD_ID="{build_id}"'] if src == "api.cpp" else [])
        unit_id = _digest([os.path.join(CSRC, src)] + headers, " ".join(flags))
        if incremental and os.path.exists(obj) and os.path.exists(stamp) and open(stamp).read() == unit_id:
            return obj
        cmd = [hipcc, *flags, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        with open(stamp, "w") as f:
            f.write(unit_id)
        return obj

    with ThreadPoolExecutor(max_workers=min(os.cpu_count() or 8, 16, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


def require_current() -> None:
    """Load what is built; build only if nothing is; refuse a library that is older than the sources."""
    if not os.path.exists(LIB):
        build()
    elif stale():
        raise RuntimeError(f"{LIB} was built from other sources than the tree holds (library {built_id() or 'without id'}, "
                           f"sources {source_id()}): run `python -m paper_2411_16127_amd.build` first")


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, incremental="--incremental" in sys.argv))
