"""Oracle for the mask updates of the pruning phases.  TEST INFRASTRUCTURE ONLY.

Magnitude-based weight pruning (paper Section 4, "Weight growth & pruning", the policy that sets Msk(w) = 0):
a connection is pruned iff its magnitude is at or below the (100 p_w)-th percentile of the magnitudes.
Readings taken where the paper leaves the policy open:
  * the population of the percentile is the set of connections that are still active (mask 1), so that every
    iteration of the iterative process removes the fraction p_w of what is left;
  * the (100 p)-th percentile of n values is the k-th smallest with k = ceil(p n) (k = 0: nothing is pruned);
  * ties with the threshold are pruned together (the policy says "less than or equal").

Row/column pruning (the paper's row/column pruning algorithm): importance of a row / column is the sum of the
magnitudes of its effective weights; the thresholds are the (p_r M)-th smallest row sum and the (p_c N)-th smallest
column sum (the listing names them the other way round in its loops and scales the row count by the column count;
a threshold for rows can only be a row-sum order statistic counted in rows, which is the reading here), both taken
before anything is removed; then rows at or below the row threshold are zeroed (mask and weights), and then columns
whose sum over the matrix as the row loop left it is at or below the column threshold.  k = ceil(p * count);
k = 0 removes nothing along that axis.

Sums: each row / column sum is accumulated in float64 in index order, s = (((0 + e_0) + e_1) + ...) + e_last with
e_k = |w| for an active entry and 0 otherwise (written as an explicit loop below; numpy's own sum is pairwise and
would round differently).  The paper's algorithm does not give an order; one has to be fixed because a float64 sum
of thousands of float32 magnitudes is not exact, and the order-statistic comparison that follows decides whole rows
and columns.
"""
from __future__ import annotations

import math
from typing import Tuple

import numpy as np


def prune_weights(W: np.ndarray, mask: np.ndarray, p_w: float) -> np.ndarray:
    """New mask after one magnitude-pruning iteration with ratio p_w."""
    W = np.asarray(W, dtype=np.float32)
    mask = np.asarray(mask, dtype=np.uint8)
    active = np.flatnonzero(mask.ravel())
    k = math.ceil(p_w * active.size)
    out = mask.copy()
    if k <= 0:
        return out
    mags = np.abs(W.ravel()[active])
    thr = np.sort(mags, kind="stable")[k - 1]
    flat = out.ravel()
    flat[active[mags <= thr]] = 0
    return out


def _row_sums_in_index_order(eff: np.ndarray) -> np.ndarray:
    acc = np.zeros(eff.shape[0], np.float64)
    for k in range(eff.shape[1]):        # column after column: every row's sum grows by its k-th entry
        acc = acc + eff[:, k]
    return acc


def _col_sums_in_index_order(eff: np.ndarray) -> np.ndarray:
    acc = np.zeros(eff.shape[1], np.float64)
    for r in range(eff.shape[0]):
        acc = acc + eff[r, :]
    return acc


def prune_rows_cols_lines(W: np.ndarray, mask: np.ndarray, p_r: float, p_c: float) -> Tuple[np.ndarray, np.ndarray]:
    """Which rows and which columns one row/column pruning iteration removes (two boolean vectors)."""
    W = np.asarray(W, dtype=np.float32)
    mask = np.asarray(mask, dtype=np.uint8)
    M, N = W.shape
    eff = np.where(mask == 1, np.abs(W).astype(np.float64), 0.0)
    row_sum = _row_sums_in_index_order(eff)
    col_sum = _col_sums_in_index_order(eff)
    kr, kc = math.ceil(p_r * M), math.ceil(p_c * N)
    rows = np.zeros(M, bool)
    cols = np.zeros(N, bool)
    if kr > 0:
        th_r = np.sort(row_sum)[kr - 1]
        rows = row_sum <= th_r
    if kc > 0:
        th_c = np.sort(col_sum)[kc - 1]          # threshold of the matrix as passed in
        eff[rows, :] = 0.0                       # the column loop sees what the row loop left
        cols = _col_sums_in_index_order(eff) <= th_c
    return rows, cols


def prune_rows_cols(W: np.ndarray, mask: np.ndarray, p_r: float, p_c: float) -> Tuple[np.ndarray, np.ndarray]:
    """(W, mask) after one row/column pruning iteration: the removed lines are zeroed in both."""
    W = np.array(W, dtype=np.float32, copy=True)
    mask = np.array(mask, dtype=np.uint8, copy=True)
    rows, cols = prune_rows_cols_lines(W, mask, p_r, p_c)
    mask[rows, :] = 0
    W[rows, :] = 0.0
    mask[:, cols] = 0
    W[:, cols] = 0.0
    return W, mask
