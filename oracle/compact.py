"""Oracle for dimension compaction after row/column pruning.  TEST INFRASTRUCTURE ONLY.

Row/column pruning shrinks the dimensions of a weight matrix (paper Section 4, "Row/column growth & pruning";
Section 5.1 step (b): each control-gate matrix goes from 1500/400 to 1197/317; Section 5.2 step (b): 800/800 to
626/626): rows and columns whose connections have all been pruned away leave the matrix, and what is left is a smaller
dense matrix.  The definition written out:

  * the matrix holds `gates` blocks of R rows, one block per control gate (row q*R + r is unit r of gate q); a unit is
    kept iff at least one of its `gates` rows has an active connection (mask byte 1), so that the blocks keep a common
    height (a neuron goes when all of its input connections are gone - Section 4, weight pruning paragraph);
  * a column is kept iff at least one row has an active connection in it;
  * kept units and kept columns keep their order;
  * the compacted matrix has gates*Rc rows (same block layout) and Nc columns and holds W where the mask byte is 1 and
    +0 where it is 0 (selection, not multiplication: what lies under a zero mask byte is never looked at).

A unit or column that is dropped has no active connection, so nothing that is kept changes: the step is its own fixed
point.  Plain numpy, in index order.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def compact_rows_cols(W: np.ndarray, mask: np.ndarray, gates: int = 1) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """(row_index [Rc], col_index [Nc], Wc [gates*Rc, Nc] float32, mask_c [gates*Rc, Nc] uint8)."""
    W = np.asarray(W, dtype=np.float32)
    mask = np.asarray(mask, dtype=np.uint8)
    M, N = W.shape
    assert mask.shape == (M, N) and gates >= 1 and M % gates == 0
    R = M // gates
    active = mask == 1
    unit_kept = np.zeros(R, dtype=bool)
    for q in range(gates):
        unit_kept |= active[q * R:(q + 1) * R, :].any(axis=1)
    col_kept = active.any(axis=0)
    row_index = np.flatnonzero(unit_kept).astype(np.int32)
    col_index = np.flatnonzero(col_kept).astype(np.int32)
    Rc, Nc = row_index.size, col_index.size
    Wc = np.zeros((gates * Rc, Nc), dtype=np.float32)
    mc = np.zeros((gates * Rc, Nc), dtype=np.uint8)
    for q in range(gates):
        for i, r in enumerate(row_index):
            src_m = active[q * R + r, col_index]
            src_w = W[q * R + r, col_index]
            Wc[q * Rc + i, :] = np.where(src_m, src_w, np.float32(0.0))
            mc[q * Rc + i, :] = src_m
    return row_index, col_index, Wc, mc
