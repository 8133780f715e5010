"""Host-side byte models of bench.py (no GPU): the gather model per edge and the compulsory floor."""
import types

import bench


def fake(model, H, D, dtype, n, nnz):
    w = types.SimpleNamespace(model=model, H=H, D=D, dtype=dtype)
    g = types.SimpleNamespace(n=n, nnz=nnz)
    return w, g


def per_edge(model, H, D, dtype, edge_bias=False):
    """Bytes per edge of the three passes: the difference of the model at E + 1 and E edges."""
    w, g0 = fake(model, H, D, dtype, 1000, 5000)
    _, g1 = fake(model, H, D, dtype, 1000, 5001)
    a, b = bench.algorithmic_bytes(w, g0, edge_bias), bench.algorithmic_bytes(w, g1, edge_bias)
    return {k: b[k] - a[k] for k in ("fwd", "bwd_row", "bwd_col")}


def test_gt_moves_six_rows_per_edge():
    # forward K_j, V_j; row pass K_j, V_j; column pass Q_i, dO_i and two packed statistics per head; one index each
    for H, D, dtype, b in ((8, 16, "f32", 4), (1, 64, "f32", 4), (8, 16, "bf16", 2)):
        R, s = H * D * b, 4 * H
        e = per_edge("gt", H, D, dtype)
        assert e == {"fwd": 2 * R + 4, "bwd_row": 2 * R + 4, "bwd_col": 2 * R + 2 * s + 4}
        assert sum(e.values()) == 6 * R + 2 * s + 12


def test_one_row_models():
    R, s = 8 * 8 * 4, 32
    assert sum(per_edge("gat", 8, 8, "f32").values()) == 3 * R + 5 * s + 12
    R, s = 64 * 4, 4
    assert sum(per_edge("agnn", 1, 64, "f32").values()) == 4 * R + 5 * s + 12
    R, s = 8 * 16 * 4, 32
    assert sum(per_edge("gatv2", 8, 16, "f32").values()) == 4 * R + 2 * s + 12


def test_edge_term_adds_one_value_per_head_and_pass():
    s = 32
    plain, term = per_edge("gt", 8, 16, "f32"), per_edge("gt", 8, 16, "f32", True)
    # read by all three passes, its position read by the column pass, its gradient written once
    assert sum(term.values()) - sum(plain.values()) == 4 * s + 4


def test_compulsory_floor_is_every_array_once():
    w, g = fake("gt", 8, 16, "f32", 1000, 5000)
    T, S, csr = 1000 * 512, 1000 * 32, 4 * 1001 + 4 * 5000
    # forward: Q, K, V in, O and two statistics out, CSR; backward: Q, K, V, O, dO in, three gradients out,
    # statistics, CSR and CSC
    assert bench.compulsory_bytes(w, g) == (4 * T + 2 * S + csr) + (8 * T + 2 * S + 2 * csr)
    assert bench.compulsory_bytes(w, g) < sum(bench.algorithmic_bytes(w, g)[k] for k in ("fwd", "bwd_row", "bwd_col"))


def test_measured_traffic_is_given_only_for_the_kernel_sources_it_was_measured_on(tmp_path, monkeypatch):
    """roofline.traffic comes from a table that names the hash of the layer-kernel sources; any other hash,
    an unknown kernel or a missing table give None (the bench line then says null)."""
    from paper_2411_16127_amd.build import kernels_id
    table = tmp_path / "measured_traffic.md"
    table.write_text("| workload | kernel | bytes per launch | layer-kernel sources |\n|---|---|---|---|\n"
                     f"| cfg5 | bwd_col | 141900000000 | `{kernels_id()}` |\n"
                     "| cfg5 | fwd | 123900000000 | `0123456789abcdef01234567` |\n")
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(table))
    assert bench.measured_traffic("cfg5", "bwd_col") == 141900000000
    assert bench.measured_traffic("cfg5", "fwd") is None       # measured on other sources: stale
    assert bench.measured_traffic("cfg5", "bwd_row") is None   # not in the table
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "absent.md"))
    assert bench.measured_traffic("cfg5", "bwd_col") is None


def test_more_than_one_gpu_is_refused():
    """This build runs on one GPU: `--gpus 2` ends with a message and a non-zero status before anything is set up."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
