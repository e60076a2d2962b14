"""Oracle for the per-row compressed form of a masked weight matrix.  TEST INFRASTRUCTURE ONLY.

Mask-based approach of the paper's Section 4: the effective matrix is W (x) Msk.  The
compressed form keeps, per row, exactly the positions where Msk = 1 (whatever value W
holds there, zero included), in ascending column order.  With no mask every position is kept.
"""
import numpy as np


def row_compress(W: np.ndarray, M):
    W = np.asarray(W, dtype=np.float32)
    rows, cols = W.shape
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    col = []
    val = []
    for r in range(rows):
        for k in range(cols):
            if M is None or M[r, k] != 0:
                col.append(k)
                val.append(W[r, k])
        row_ptr[r + 1] = len(col)
    return row_ptr, np.asarray(col, dtype=np.int64), np.asarray(val, dtype=np.float32)


def masked_dense(W: np.ndarray, M):
    """W where Msk = 1, +0.0 elsewhere (a selection, so non-finite values under Msk = 0 vanish)."""
    W = np.asarray(W, dtype=np.float32)
    if M is None:
        return W.copy()
    out = np.zeros_like(W)
    keep = np.asarray(M) != 0
    out[keep] = W[keep]
    return out
