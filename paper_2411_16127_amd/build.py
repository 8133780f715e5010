"""Builds libdfgnn.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2411_16127_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
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


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel) and link the shared library."""
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=min(os.cpu_count() or 8, 16, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
