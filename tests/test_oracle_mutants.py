"""Mutation check of the oracle pins (CPU only).  Each case plants one plausible mistake (a dropped factor, a
wrong index, a missing softmax term, a wrong derivative branch, a wrong sign ...) in a copy of the oracle's C
source, builds it, and runs tests/test_oracle_pins.py against the copy in a child process (tests/pins_against_copy.py): at least one pin must
fail for every mutant, and all pins must pass for the unchanged copy."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "atgnn_oracle.c")
# the copy is put in place by the child process itself (test side); the oracle package has no switch for it
RUNNER = os.path.join(ROOT, "tests", "pins_against_copy.py")

MUTANTS = [
    # GT: score scale dropped from dQ; dK reads the wrong row of Q
    ("dX[(i * H + h) * D + d] += L->scale * dS * K", "dX[(i * H + h) * D + d] += dS * K"),
    ("dK[(j * H + h) * D + d] += L->scale * dS * X[(i", "dK[(j * H + h) * D + d] += L->scale * dS * X[(j"),
    # softmax backward without its row term; softmax without the maximum shift (overflows at large scores)
    ("const double dS = p[t - b] * (dP[t - b] - pdp);", "const double dS = p[t - b] * (dP[t - b]);"),
    ("p[t - b] = exp(p[t - b] - m);", "p[t - b] = exp(p[t - b]);"),
    # GAT: LeakyReLU derivative and value, the source-side gradient on the wrong node, a_r / a_l mixed up
    ("gat_z(&c, i, j, h) > 0.0 ? 1.0 : L->neg_slope", "1.0"),
    ("return z > 0.0 ? z : c->L->neg_slope * z;", "return z > 0.0 ? z : z;"),
    ("d_er[j * H + h] += dz;", "d_er[i * H + h] += dz;"),
    ("c->er[v * H + h] = dot(a_r + h * D, x, D);", "c->er[v * H + h] = dot(a_l + h * D, x, D);"),
    ("da_r[h * D + d] += d_er[v", "da_r[h * D + d] += d_el[v"),
    # AGNN: the wrong feature row in the source-side gradient, no projection in the norm backward, dbeta without c_ij
    ("g[(j * H + h) * D + d] += L->scale * dS * xi[d];", "g[(j * H + h) * D + d] += L->scale * dS * xj[d];"),
    ("(gv[d] - proj * xh[d]) / c.nrm", "(gv[d]) / c.nrm"),
    ("*dscale += dS * dot(xi, xj, D);", "*dscale += dS;"),
    # GATv2: no LeakyReLU in the score, source and destination swapped, derivative branch, gradient rows
    ("s += c->a[h * D + d] * (z > 0.0 ? z : c->L->neg_slope * z);", "s += c->a[h * D + d] * z;"),
    ("const double z = c->X[(i * H + h) * D + d] + c->K[(j * H + h) * D + d];",
     "const double z = c->X[(j * H + h) * D + d] + c->K[(i * H + h) * D + d];"),
    ("const double dz = dS * a_l[h * D + d] * (z > 0.0 ? 1.0 : L->neg_slope);", "const double dz = dS * a_l[h * D + d];"),
    ("dK[(j * H + h) * D + d] += dz;", "dK[(i * H + h) * D + d] += dz;"),
    ("da_l[h * D + d] += dS * (z > 0.0 ? z : L->neg_slope * z);", "da_l[h * D + d] += dS * z;"),
    ("da_l[h * D + d] += dS * (z > 0.0 ? z : L->neg_slope * z);", "da_l[h * D + d] += dz;"),
    ("(L->model == ATGNN_GATV2 ? dK : dX);", "dX;"),
    ("(L->model == ATGNN_GATV2 ? K : X);", "X;"),
    # edge term: wrong sign, wrong head, ignored
    ("return c->bias ? s + c->bias[t * c->L->H + h] : s;", "return c->bias ? s - c->bias[t * c->L->H + h] : s;"),
    ("return c->bias ? s + c->bias[t * c->L->H + h] : s;", "return c->bias ? s + c->bias[t * c->L->H] : s;"),
    ("return c->bias ? s + c->bias[t * c->L->H + h] : s;", "return s;"),
]


def pins_pass(source: str, workdir, tag: str) -> bool:
    c_file = os.path.join(workdir, f"oracle_{tag}.c")
    lib = os.path.join(workdir, f"liboracle_{tag}.so")
    with open(c_file, "w") as f:
        f.write(source)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-w", "-o", lib, c_file, "-lm"])
    run = subprocess.run([sys.executable, RUNNER, "layer", lib], cwd=ROOT, stdout=subprocess.DEVNULL,
                         stderr=subprocess.DEVNULL)
    return run.returncode == 0


def test_every_planted_mistake_fails_a_pin(tmp_path):
    original = open(SRC).read()
    for old, _ in MUTANTS:
        assert original.count(old) == 1, f"the oracle no longer contains: {old}"
    assert pins_pass(original, str(tmp_path), "unchanged")
    with ThreadPoolExecutor(max_workers=4) as pool:
        survived = list(pool.map(lambda m: pins_pass(original.replace(m[1][0], m[1][1]), str(tmp_path), str(m[0])),
                                 enumerate(MUTANTS)))
    assert not any(survived), [MUTANTS[i] for i, s in enumerate(survived) if s]


SCHED_SRC = os.path.join(ROOT, "oracle", "sched_oracle.py")
SCHED_MUTANTS = [
    # super rows from T + 1 instead of T (in the sort key; in the count)
    ("key = np.where(deg >= T, 0, 33 - _bit_length(deg))", "key = np.where(deg > T, 0, 33 - _bit_length(deg))"),
    ("n_super = int(np.count_nonzero(deg >= T))", "n_super = int(np.count_nonzero(deg > T))"),
    # equal keys in descending instead of ascending id order (rows; CSC entries)
    ('order = np.argsort(key, kind="stable")',
     'order = np.argsort(key)[::-1][np.argsort(key[np.argsort(key)[::-1]], kind="stable")]'),
    ('t_eid = np.argsort(indices, kind="stable")',
     't_eid = np.argsort(indices, kind="stable")[::-1][np.argsort(indices[np.argsort(indices, kind="stable")[::-1]], kind="stable")]'),
    # chunk count rounded down; last chunk not clipped; chunk stride off by one; short rows before long ones
    ("n_chunks = -(-deg[sup] // C)", "n_chunks = deg[sup] // C"),
    ("chunks[pos] = (row, b, min(b + C, indptr[row + 1]))", "chunks[pos] = (row, b, b + C)"),
    ("b = indptr[row] + c * C", "b = indptr[row] + c * (C - 1)"),
    ("33 - _bit_length(deg)", "_bit_length(deg)"),
    # CSC lists sources instead of destinations
    ('"t_indices": rows[t_eid]', '"t_indices": indices[t_eid]'),
]


def sched_pins_pass(source: str, workdir, tag: str) -> bool:
    py_file = os.path.join(workdir, f"sched_oracle_{tag}.py")
    with open(py_file, "w") as f:
        f.write(source)
    run = subprocess.run([sys.executable, RUNNER, "sched", py_file], cwd=ROOT, stdout=subprocess.DEVNULL,
                         stderr=subprocess.DEVNULL)
    return run.returncode == 0


def test_every_planted_mistake_in_the_metadata_oracle_fails_a_pin(tmp_path):
    original = open(SCHED_SRC).read()
    for old, _ in SCHED_MUTANTS:
        assert original.count(old) >= 1, f"the metadata oracle no longer contains: {old}"
    assert sched_pins_pass(original, str(tmp_path), "unchanged")
    with ThreadPoolExecutor(max_workers=4) as pool:
        survived = list(pool.map(lambda m: sched_pins_pass(original.replace(m[1][0], m[1][1]), str(tmp_path), str(m[0])),
                                 enumerate(SCHED_MUTANTS)))
    assert not any(survived), [SCHED_MUTANTS[i] for i, s in enumerate(survived) if s]
