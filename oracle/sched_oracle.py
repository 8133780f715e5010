"""Integer oracle for the scheduling metadata of a CSR graph (test infrastructure only).

The fused layer switches work mapping by neighbourhood size (Sec. 4.2, the super-node condition of
the SDDMM paragraph); here the switch is per row.  This file states the metadata contract in the
plainest form available (numpy stable sorts); the HIP library must reproduce it bit for bit.

Contract, for degree array deg, threshold T (rows with deg >= T are 'super') and chunk size C:
  bucket(i)  = bit_length(deg[i])                      (0 for an empty row)
  key(i)     = 0 if deg[i] >= T else 33 - bucket(i)    (super rows first, then long rows before short)
  order      = stable ascending sort of row ids by key
  n_super    = number of super rows (they are order[:n_super], ascending ids)
  chunk_ptr  = exclusive prefix sum of ceil(deg/C) over the super rows in that order  [n_super+1]
  chunks     = for each super row in that order, c = 0..ceil(deg/C)-1:
               (row, begin = indptr[row] + c*C, end = min(begin + C, indptr[row+1]))
CSC transpose: out-edges of source j listed in increasing CSR edge position:
  t_indptr[j+1]-t_indptr[j] = out-degree of j;  t_eid = CSR positions, ascending inside a column;
  t_indices[e'] = destination row of CSR edge t_eid[e'].
"""
from __future__ import annotations

from typing import Dict

import numpy as np


def _bit_length(deg: np.ndarray) -> np.ndarray:
    out = np.zeros(deg.shape, dtype=np.int64)
    d = deg.astype(np.int64).copy()
    while np.any(d > 0):
        out += d > 0
        d >>= 1
    return out


def schedule(indptr: np.ndarray, T: int, C: int) -> Dict[str, np.ndarray]:
    """Row order and super-row chunks for one CSR-like pointer array (rows or, for the CSC, columns)."""
    indptr = np.asarray(indptr, dtype=np.int64)
    n = indptr.size - 1
    deg = np.diff(indptr)
    key = np.where(deg >= T, 0, 33 - _bit_length(deg))
    order = np.argsort(key, kind="stable")
    n_super = int(np.count_nonzero(deg >= T))
    sup = order[:n_super]
    n_chunks = -(-deg[sup] // C)
    chunk_ptr = np.zeros(n_super + 1, dtype=np.int64)
    np.cumsum(n_chunks, out=chunk_ptr[1:])
    chunks = np.zeros((int(chunk_ptr[-1]), 3), dtype=np.int64)
    pos = 0
    for s in range(n_super):
        row = int(sup[s])
        for c in range(int(n_chunks[s])):
            b = indptr[row] + c * C
            chunks[pos] = (row, b, min(b + C, indptr[row + 1]))
            pos += 1
    return {"order": order.astype(np.int32), "n_super": n_super, "chunk_ptr": chunk_ptr.astype(np.int32),
            "chunks": chunks.astype(np.int32)}


def csc_transpose(indptr: np.ndarray, indices: np.ndarray) -> Dict[str, np.ndarray]:
    indptr = np.asarray(indptr, dtype=np.int64)
    indices = np.asarray(indices, dtype=np.int64)
    n = indptr.size - 1
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(indptr))
    t_eid = np.argsort(indices, kind="stable")
    t_indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(indices, minlength=n), out=t_indptr[1:])
    return {"t_indptr": t_indptr.astype(np.int32), "t_indices": rows[t_eid].astype(np.int32),
            "t_eid": t_eid.astype(np.int32)}
