"""Helper shared by the compaction tests: apply a compaction routine to every matrix of a plain-LSTM case and build
the case of the compacted model.  `compact(W, mask, gates)` is the routine under test (the oracle's, or a wrapper
round the library's) and returns (row_index, col_index, Wc, mask_c)."""
from __future__ import annotations

from dataclasses import replace

import numpy as np

from paper_1901_10997_amd import inputs


def compact_case(case, compact):
    """(compacted case, units[(l, d)], feats[, gate_units[(l, d)]]): every layer and direction must come out with the
    same number of units, a recurrent matrix must keep exactly the columns of its own units, and an upper layer's
    input matrix exactly the units the layer below kept - the conditions under which dropping them changes nothing
    that is kept.  H-LSTM cases: the hidden layers inside the gates are compacted too (rows of the two first-stage
    matrices, columns of the gate-output matrix)."""
    w = case.w
    H, G = w.hidden, w.gate_hidden
    units, gate_units, weights = {}, {}, {}
    feats = None
    for l in range(w.layers):
        for d in range(w.ndir):
            cur = case.weights[(l, d)]
            if G > 0:
                rx, cx, Wxc, Mxc = compact(cur["W1x"], cur["M1x"], 4)
                r1, ch, Whc, Mhc = compact(cur["W1h"], cur["M1h"], 4)
                rh, c2, W2c, M2c = compact(cur["W2"], cur["M2"], 4)
                np.testing.assert_array_equal(rx, r1)
                np.testing.assert_array_equal(c2, r1)
                gate_units[(l, d)] = np.asarray(r1)
            else:
                rx, cx, Wxc, Mxc = compact(cur["Wx"], cur["Mx"], 4)
                rh, ch, Whc, Mhc = compact(cur["Wh"], cur["Mh"], 4)
                np.testing.assert_array_equal(rx, rh)
            np.testing.assert_array_equal(ch, rh)
            if l == 0:
                if feats is None:
                    feats = np.asarray(cx)
                np.testing.assert_array_equal(cx, feats)
            else:
                below = np.concatenate([dd * H + units[(l - 1, dd)] for dd in range(w.ndir)])
                np.testing.assert_array_equal(cx, below)
            units[(l, d)] = np.asarray(rh)
            if G > 0:
                b1 = np.ascontiguousarray(cur["b1"].reshape(4, G)[:, r1].reshape(-1))
                b2 = np.ascontiguousarray(cur["b2"].reshape(4, H)[:, rh].reshape(-1))
                weights[(l, d)] = dict(W1x=Wxc, M1x=Mxc, W1h=Whc, M1h=Mhc, b1=b1, W2=W2c, M2=M2c, b2=b2)
            else:
                b4 = cur["b"].reshape(4, H)[:, rh].reshape(-1)
                weights[(l, d)] = dict(Wx=Wxc, Mx=Mxc, Wh=Whc, Mh=Mhc, b=np.ascontiguousarray(b4))
    sizes = {len(u) for u in units.values()}
    assert len(sizes) == 1
    Hc = sizes.pop()
    gsizes = {len(u) for u in gate_units.values()}
    assert len(gsizes) <= 1
    wc = replace(w, hidden=Hc, input_dim=len(feats), gate_hidden=gsizes.pop() if gsizes else 0)
    x = np.ascontiguousarray(case.x[:, :, feats])

    def state(s):
        if s is None:
            return None
        out = np.zeros((w.layers * w.ndir, w.B, Hc), np.float32)
        for l in range(w.layers):
            for d in range(w.ndir):
                out[l * w.ndir + d] = s[l * w.ndir + d][:, units[(l, d)]]
        return out

    small = inputs.Case(wc, case.seed, weights, x, state(case.h0), state(case.c0))
    if G > 0:
        return small, units, feats, gate_units
    return small, units, feats


def restrict_outputs(ref, w, units):
    """(y, hT, cT) of the full model at the units the compacted model keeps."""
    y, hT, cT = ref
    H = w.hidden
    last = w.layers - 1
    ycols = np.concatenate([d * H + units[(last, d)] for d in range(w.ndir)])
    Hc = len(units[(0, 0)])
    h = np.zeros((w.layers * w.ndir, y.shape[1], Hc))
    c = np.zeros_like(h)
    for l in range(w.layers):
        for d in range(w.ndir):
            h[l * w.ndir + d] = hT[l * w.ndir + d][:, units[(l, d)]]
            c[l * w.ndir + d] = cT[l * w.ndir + d][:, units[(l, d)]]
    return y[:, :, ycols], h, c
