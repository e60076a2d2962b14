"""Pins of the dimension-compaction oracle (no GPU): a hand example, brute force in plain loops, the product identity
that defines a correct compaction, its fixed point, and the model-level statement that a compacted LSTM computes what
the row/column-pruned one computes at the units that are kept."""
import numpy as np
import pytest

from compact_util import compact_case, restrict_outputs
from oracle import compact as ocompact
from oracle import lstm_oracle as orc
from paper_1901_10997_amd import inputs


def test_hand_example_one_gate():
    W = np.array([[1.0, 2.0, 3.0, 4.0],
                  [5.0, 6.0, 7.0, 8.0],
                  [9.0, 1.5, 2.5, 3.5]], np.float32)
    m = np.array([[1, 0, 0, 1],
                  [0, 0, 0, 0],
                  [0, 0, 1, 1]], np.uint8)
    r, c, Wc, mc = ocompact.compact_rows_cols(W, m, 1)
    np.testing.assert_array_equal(r, [0, 2])          # row 1 has no connection left
    np.testing.assert_array_equal(c, [0, 2, 3])       # column 1 neither
    np.testing.assert_array_equal(Wc, [[1.0, 0.0, 4.0], [0.0, 2.5, 3.5]])
    np.testing.assert_array_equal(mc, [[1, 0, 1], [0, 1, 1]])
    assert Wc.dtype == np.float32 and mc.dtype == np.uint8 and r.dtype == np.int32 and c.dtype == np.int32


def test_hand_example_gate_blocks_keep_a_common_height():
    # two gates of three units: unit 1 is dead in gate 0 but alive in gate 1 -> kept in both (a zero row in gate 0);
    # unit 2 is dead in both -> dropped from both
    W = np.arange(1, 13, dtype=np.float32).reshape(6, 2)
    m = np.array([[1, 0], [0, 0], [0, 0],
                  [0, 0], [1, 0], [0, 0]], np.uint8)
    r, c, Wc, mc = ocompact.compact_rows_cols(W, m, 2)
    np.testing.assert_array_equal(r, [0, 1])
    np.testing.assert_array_equal(c, [0])
    np.testing.assert_array_equal(Wc, [[1.0], [0.0], [0.0], [9.0]])
    np.testing.assert_array_equal(mc, [[1], [0], [0], [1]])


def test_values_under_a_zero_mask_byte_are_never_looked_at():
    W = np.array([[np.nan, 2.0], [np.inf, -np.inf]], np.float32)
    m = np.array([[0, 1], [0, 0]], np.uint8)
    r, c, Wc, mc = ocompact.compact_rows_cols(W, m, 1)
    np.testing.assert_array_equal(r, [0]); np.testing.assert_array_equal(c, [1])
    np.testing.assert_array_equal(Wc, [[2.0]])
    # an active connection whose weight is zero is still a connection
    r, c, Wc, mc = ocompact.compact_rows_cols(np.zeros((2, 2), np.float32), np.array([[0, 0], [1, 0]], np.uint8), 1)
    np.testing.assert_array_equal(r, [1]); np.testing.assert_array_equal(c, [0])
    assert Wc.shape == (1, 1) and Wc[0, 0] == 0.0 and not np.signbit(Wc[0, 0]) and mc[0, 0] == 1


def test_full_and_empty_masks():
    rng = np.random.default_rng(0)
    W = rng.standard_normal((8, 5)).astype(np.float32)
    r, c, Wc, mc = ocompact.compact_rows_cols(W, np.ones((8, 5), np.uint8), 4)
    np.testing.assert_array_equal(r, [0, 1]); np.testing.assert_array_equal(c, np.arange(5))
    np.testing.assert_array_equal(Wc, W); assert mc.all()
    r, c, Wc, mc = ocompact.compact_rows_cols(W, np.zeros((8, 5), np.uint8), 4)
    assert r.size == 0 and c.size == 0 and Wc.shape == (0, 0) and mc.shape == (0, 0)


def _structured(rng, gates, R, N, keep):
    M = gates * R
    W = rng.standard_normal((M, N)).astype(np.float32)
    m = (rng.random((M, N)) < keep).astype(np.uint8)
    dead_units = rng.random(R) < 0.3
    dead_cols = rng.random(N) < 0.3
    m[np.tile(dead_units, gates), :] = 0
    m[:, dead_cols] = 0
    return W, m


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_in_plain_loops(seed):
    rng = np.random.default_rng(10 + seed)
    gates, R, N = int(rng.integers(1, 5)), int(rng.integers(1, 7)), int(rng.integers(1, 9))
    W, m = _structured(rng, gates, R, N, 0.4)
    r, c, Wc, mc = ocompact.compact_rows_cols(W, m, gates)
    rows = [u for u in range(R) if any(m[q * R + u, k] for q in range(gates) for k in range(N))]
    cols = [k for k in range(N) if any(m[i, k] for i in range(gates * R))]
    assert list(r) == rows and list(c) == cols
    assert Wc.shape == (gates * len(rows), len(cols)) == mc.shape
    for q in range(gates):
        for i, u in enumerate(rows):
            for j, k in enumerate(cols):
                src = (q * R + u, k)
                assert mc[q * len(rows) + i, j] == m[src]
                assert Wc[q * len(rows) + i, j] == (W[src] if m[src] else 0.0)


@pytest.mark.parametrize("seed", range(4))
def test_product_identity_and_fixed_point(seed):
    """(W (.) Msk) x, taken at the kept rows, equals Wc x[kept columns]; dropped rows give exactly zero; compacting the
    compacted matrix changes nothing."""
    rng = np.random.default_rng(50 + seed)
    gates, R, N = 4, 37, 53
    W, m = _structured(rng, gates, R, N, 0.3)
    r, c, Wc, mc = ocompact.compact_rows_cols(W, m, gates)
    eff = np.where(m == 1, W.astype(np.float64), 0.0)
    x = rng.standard_normal(N)
    full = eff @ x
    kept_rows = np.concatenate([q * R + r for q in range(gates)])
    np.testing.assert_allclose(Wc.astype(np.float64) @ x[c], full[kept_rows], rtol=0, atol=1e-12)
    dropped = np.setdiff1d(np.arange(gates * R), kept_rows)
    assert dropped.size > 0 and np.all(full[dropped] == 0.0)
    assert 0 < r.size < R and 0 < c.size < N
    r2, c2, Wc2, mc2 = ocompact.compact_rows_cols(Wc, mc, gates)
    np.testing.assert_array_equal(r2, np.arange(r.size)); np.testing.assert_array_equal(c2, np.arange(c.size))
    np.testing.assert_array_equal(Wc2, Wc); np.testing.assert_array_equal(mc2, mc)
    # counts: no active connection is lost
    assert int(mc.sum()) == int(m.sum())


@pytest.mark.parametrize("bidir,layers", [(False, 1), (False, 2), (True, 2)])
def test_compacted_lstm_computes_the_pruned_models_outputs(bidir, layers):
    """The paper's row/column-pruned model and the smaller dense-dimension model are the same function at the kept
    units (Section 5.1 step (b): 1500/400 -> 1197/317): checked with the forward oracle on both."""
    w = inputs.shrink(inputs.c2(2), layers=layers, bidirectional=bidir, input_dim=20, hidden=24, T=6, B=2, keep=0.6,
                      bias="uniform", a=0.4)
    case = inputs.make_case(w, k=3, random_state=True)
    pruned, units, feats = inputs.structure_masks(case, 0.75, 0.8, k=1)
    small, found_units, found_feats = compact_case(pruned, ocompact.compact_rows_cols)
    np.testing.assert_array_equal(found_feats, feats)
    for key in units:
        np.testing.assert_array_equal(found_units[key], units[key])
    assert small.w.hidden == 18 and small.w.input_dim == 16
    ref = restrict_outputs(orc.forward_case(pruned), w, units)
    got = orc.forward_case(small)
    for a, b in zip(got, ref):
        assert a.shape == b.shape
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
    # and the kept units do depend on what was kept: the unpruned model gives something else
    other = restrict_outputs(orc.forward_case(case), w, units)
    assert np.max(np.abs(other[0] - ref[0])) > 1e-3


@pytest.mark.parametrize("bidir,layers", [(False, 1), (True, 2)])
def test_compacted_hlstm_computes_the_pruned_models_outputs(bidir, layers):
    """The same statement for the H-LSTM cell: hidden units, input features and the hidden-layer units inside the gates
    all leave, and the kept outputs do not change."""
    from oracle import hlstm_oracle as horc
    w = inputs.shrink(inputs.h1(), layers=layers, bidirectional=bidir, input_dim=20, hidden=24, gate_hidden=28, T=5, B=2,
                      keep=0.6, a=0.4)
    case = inputs.make_case(w, k=4, random_state=True)
    pruned, units, feats, gunits = inputs.structure_masks(case, 0.75, 0.8, k=3, gate_unit_frac=0.5)
    small, found_units, found_feats, found_gunits = compact_case(pruned, ocompact.compact_rows_cols)
    np.testing.assert_array_equal(found_feats, feats)
    for key in units:
        np.testing.assert_array_equal(found_units[key], units[key])
        np.testing.assert_array_equal(found_gunits[key], gunits[key])
    assert (small.w.hidden, small.w.input_dim, small.w.gate_hidden) == (18, 16, 14)
    ref = restrict_outputs(horc.forward_case(pruned), w, units)
    got = horc.forward_case(small)
    for a, b in zip(got, ref):
        assert a.shape == b.shape
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
    other = restrict_outputs(horc.forward_case(case), w, units)
    assert np.max(np.abs(other[0] - ref[0])) > 1e-3
