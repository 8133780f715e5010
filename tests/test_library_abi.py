"""Host-side checks that need no GPU: the library loads, exports every declared symbol, and its
host-only entry points validate their arguments."""
import os
import re

import pytest

import paper_2411_16127_amd as dfgnn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dfgnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dfgnn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert {"dfgnn_graph_create", "dfgnn_forward", "dfgnn_backward", "dfgnn_workspace_bytes"} <= set(names)
    L = dfgnn.lib()
    for name in names:
        assert hasattr(L, name), name


def test_version_and_status_strings():
    assert dfgnn.version() == (0, 1)
    for code in range(5):
        assert dfgnn.status_string(code).startswith("DFGNN_")
    assert "unknown" in dfgnn.status_string(99)


def test_meta_bytes_validation_and_growth():
    small = dfgnn.graph_meta_bytes(100, 1000)
    big = dfgnn.graph_meta_bytes(100, 100000)
    assert big[0] > small[0] and big[1] > small[1]
    assert dfgnn.graph_meta_bytes(0, 0)[0] > 0
    with pytest.raises(dfgnn.DfgnnError) as e:
        dfgnn.graph_meta_bytes(-1, 10)
    assert e.value.status == 1
    with pytest.raises(dfgnn.DfgnnError) as e:
        dfgnn.graph_meta_bytes(10, 2**31)
    assert e.value.status == 2
    with pytest.raises(dfgnn.DfgnnError) as e:
        dfgnn.graph_meta_bytes(10, 10, dfgnn.SchedParams(-5, 1))
    assert e.value.status == 1


def test_oracle_is_not_reachable_from_the_product_package():
    pkg = os.path.join(ROOT, "paper_2411_16127_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_layer_calls_reject_missing_handles_before_touching_the_gpu():
    """NULL graph or layer: EINVAL from the host-side checks (no GPU needed), with a message."""
    import ctypes
    L = dfgnn.lib()
    null = ctypes.c_void_p(None)
    sz = ctypes.c_size_t()
    calls = {
        "dfgnn_workspace_bytes": (null, null, ctypes.byref(sz), ctypes.byref(sz)),
        "dfgnn_forward": (null, null) + (null,) * 8 + (null, 0, null),
        "dfgnn_forward_edge_bias": (null, null) + (null,) * 9 + (null, 0, null),
        "dfgnn_backward": (null, null) + (null,) * 15 + (null, 0, null),
        "dfgnn_backward_edge_bias": (null, null) + (null,) * 17 + (null, 0, null),
        "dfgnn_attention_weights": (null, null) + (null,) * 8 + (null,),
    }
    for name, args in calls.items():
        assert getattr(L, name)(*args) == 1, name  # DFGNN_EINVAL
        assert "NULL" in dfgnn.last_error(), name
