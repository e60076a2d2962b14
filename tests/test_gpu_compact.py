"""GPU parity of the dimension compaction against the numpy oracle (bit-exact: indices, mask bytes and copied weights),
and the end-to-end use: a row/column-pruned LSTM, compacted on the device, run at its smaller dimensions."""
import numpy as np
import pytest

from compact_util import compact_case, restrict_outputs
from oracle import compact as ocompact
from oracle import lstm_oracle as orc
from paper_1901_10997_amd import binding as B
from paper_1901_10997_amd import inputs
from parity_util import compare, run_gpu

pytestmark = pytest.mark.gpu


def gpu_compact(W, mask, gates):
    """The library's compaction on host arrays: (row_index, col_index, Wc, mask_c) trimmed to what was kept, after
    checking the parts of the output buffers that the call must fill with -1 or leave alone."""
    import torch
    W = np.ascontiguousarray(W, np.float32)
    mask = np.ascontiguousarray(mask, np.uint8)
    M, N = W.shape
    R = M // gates
    dev = torch.device("cuda:0")
    dW, dm = torch.from_numpy(W).to(dev), torch.from_numpy(mask).to(dev)
    ri = torch.full((R,), 12345, dtype=torch.int32, device=dev)
    ci = torch.full((N,), 12345, dtype=torch.int32, device=dev)
    Wc = torch.full((M * N,), -7.0, dtype=torch.float32, device=dev)
    mc = torch.full((M * N,), 9, dtype=torch.uint8, device=dev)
    Rc, Nc = B.lstm_compact_rows_cols(dW.data_ptr(), dm.data_ptr(), gates, R, N, ri.data_ptr(), ci.data_ptr(), Wc.data_ptr(),
                                      mc.data_ptr())
    ri, ci, Wc, mc = ri.cpu().numpy(), ci.cpu().numpy(), Wc.cpu().numpy(), mc.cpu().numpy()
    assert np.all(ri[Rc:] == -1) and np.all(ci[Nc:] == -1)
    n = gates * Rc * Nc
    assert np.all(Wc[n:] == -7.0) and np.all(mc[n:] == 9)           # nothing beyond the compacted matrix is touched
    np.testing.assert_array_equal(dW.cpu().numpy(), W)               # inputs are read only
    np.testing.assert_array_equal(dm.cpu().numpy(), mask)
    return ri[:Rc], ci[:Nc], Wc[:n].reshape(gates * Rc, Nc), mc[:n].reshape(gates * Rc, Nc)


def _structured(rng, gates, R, N, keep, dead):
    M = gates * R
    W = rng.standard_normal((M, N)).astype(np.float32)
    m = (rng.random((M, N)) < keep).astype(np.uint8)
    m[np.tile(rng.random(R) < dead, gates), :] = 0
    m[:, rng.random(N) < dead] = 0
    W[m == 0] = np.float32(np.nan)                                       # never looked at
    return W, m


@pytest.mark.parametrize("gates,R,N,keep,dead,seed", [
    (1, 3, 4, 0.5, 0.3, 0), (1, 1, 1, 1.0, 0.0, 1), (4, 1, 1, 0.0, 0.0, 2), (2, 63, 65, 0.3, 0.3, 3),
    (4, 300, 257, 0.2, 0.25, 4), (1, 1025, 2049, 0.01, 0.2, 5),          # index lists longer than one pass of the scan
    (4, 1500, 400, 0.65, 0.2, 6), (4, 1500, 1500, 0.65, 0.2, 7),         # the language model's gate matrices
    (4, 800, 1600, 0.5, 0.22, 8),                                        # the speech model's input matrix
    (3, 64, 256, 1.0, 0.0, 9), (1, 4096, 3, 0.5, 0.9, 10),
])
def test_compaction_matches_oracle(gates, R, N, keep, dead, seed):
    rng = np.random.default_rng(900 + seed)
    W, m = _structured(rng, gates, R, N, keep, dead)
    got = gpu_compact(W, m, gates)
    ref = ocompact.compact_rows_cols(W, m, gates)
    for g, r, name in zip(got, ref, ("row_index", "col_index", "Wc", "mask_c")):
        assert g.shape == r.shape, name
        np.testing.assert_array_equal(g, r, err_msg=name)
    assert not np.any(np.signbit(got[2][got[3] == 0]))                   # +0 where the mask is off


def test_compaction_without_mask_output_and_fixed_point():
    import torch
    rng = np.random.default_rng(77)
    W, m = _structured(rng, 4, 50, 70, 0.4, 0.3)
    ref = ocompact.compact_rows_cols(W, m, 4)
    dev = torch.device("cuda:0")
    dW, dm = torch.from_numpy(W).to(dev), torch.from_numpy(m).to(dev)
    ri = torch.empty(50, dtype=torch.int32, device=dev)
    ci = torch.empty(70, dtype=torch.int32, device=dev)
    Wc = torch.empty(W.size, dtype=torch.float32, device=dev)
    Rc, Nc = B.lstm_compact_rows_cols(dW.data_ptr(), dm.data_ptr(), 4, 50, 70, ri.data_ptr(), ci.data_ptr(), Wc.data_ptr(), None)
    assert (Rc, Nc) == (ref[0].size, ref[1].size)
    np.testing.assert_array_equal(Wc.cpu().numpy()[:4 * Rc * Nc].reshape(4 * Rc, Nc), ref[2])
    # compacting the result keeps everything
    again = gpu_compact(ref[2], ref[3], 4)
    np.testing.assert_array_equal(again[0], np.arange(Rc)); np.testing.assert_array_equal(again[1], np.arange(Nc))
    np.testing.assert_array_equal(again[2], ref[2]); np.testing.assert_array_equal(again[3], ref[3])


def test_compaction_rejects_bad_arguments():
    import torch
    t = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    p = t.data_ptr()
    for args in [(None, p, 1, 2, 2, p, p, p, p), (p, None, 1, 2, 2, p, p, p, p), (p, p, 0, 2, 2, p, p, p, p),
                 (p, p, 1, 0, 2, p, p, p, p), (p, p, 1, 2, 0, p, p, p, p), (p, p, 1, 2, 2, None, p, p, p),
                 (p, p, 1, 2, 2, p, None, p, p), (p, p, 1, 2, 2, p, p, None, p), (p, p, 4, 1 << 20, 1 << 10, p, p, p, p)]:
        with pytest.raises(B.LstmError):
            B.lstm_compact_rows_cols(*args)


@pytest.mark.parametrize("bidir,layers,H,D,T,Bsz,uf", [
    (False, 2, 96, 40, 12, 1, 0.8),          # the language-model pattern: 1500/400 -> 1197/317 at a small size
    (True, 2, 64, 48, 9, 3, 0.78),           # bidirectional: an upper layer reads the kept units of both directions
    (False, 1, 1500, 400, 8, 1, 0.798),      # one layer at the paper's sizes: 1500/400 -> 1197/317
])
def test_pruned_model_runs_at_its_compacted_dimensions(bidir, layers, H, D, T, Bsz, uf):
    """Row/column-pruned masks -> device compaction of every matrix -> a model of the smaller dimensions, whose
    outputs match the oracle's outputs of the pruned full-size model at the kept units."""
    w = inputs.shrink(inputs.c2(Bsz), layers=layers, bidirectional=bidir, input_dim=D, hidden=H, T=T, B=Bsz, keep=0.6,
                      bias="uniform", a=min(0.4, 1.5 / np.sqrt(H)))
    case = inputs.make_case(w, k=5, random_state=True)
    pruned, units, feats = inputs.structure_masks(case, uf, 0.7925, k=2)
    small, found_units, found_feats = compact_case(pruned, gpu_compact)
    np.testing.assert_array_equal(found_feats, feats)
    for key in units:
        np.testing.assert_array_equal(found_units[key], units[key])
    if H == 1500:
        assert (small.w.hidden, small.w.input_dim) == (1197, 317)
    ref = restrict_outputs(orc.forward_case(pruned), w, units)
    gpu, desc = run_gpu(small)
    compare(gpu, ref, "f32", f"compacted {w.name} {desc}")
    # the full-size pruned model through the library gives the same (the two routes agree with each other)
    gpu_full, _ = run_gpu(pruned)
    compare(restrict_outputs(gpu_full, w, units), ref, "f32", "pruned full size")


@pytest.mark.parametrize("bidir,layers,H,G,D,T,Bsz", [
    (False, 1, 96, 80, 40, 10, 1),
    (True, 2, 64, 64, 48, 7, 4),
    (False, 1, 1500, 1500, 400, 6, 1),       # the paper's language model: 1500/400 -> 1197/317, gates' hidden layers too
])
def test_pruned_hlstm_runs_at_its_compacted_dimensions(bidir, layers, H, G, D, T, Bsz):
    from oracle import hlstm_oracle as horc
    w = inputs.shrink(inputs.h1(), layers=layers, bidirectional=bidir, input_dim=D, hidden=H, gate_hidden=G, T=T, B=Bsz,
                      keep=0.5, a=min(0.4, 1.5 / np.sqrt(max(H, G))))
    case = inputs.make_case(w, k=6, random_state=True)
    pruned, units, feats, gunits = inputs.structure_masks(case, 0.798, 0.7925, k=4)
    small, found_units, found_feats, found_gunits = compact_case(pruned, gpu_compact)
    np.testing.assert_array_equal(found_feats, feats)
    for key in units:
        np.testing.assert_array_equal(found_units[key], units[key])
        np.testing.assert_array_equal(found_gunits[key], gunits[key])
    if H == 1500:
        assert (small.w.hidden, small.w.gate_hidden, small.w.input_dim) == (1197, 1197, 317)
    ref = restrict_outputs(horc.forward_case(pruned), w, units)
    gpu, desc = run_gpu(small)
    compare(gpu, ref, "f32", f"compacted {w.name} {desc}")


@pytest.mark.parametrize("M,N,p,seed", [(320, 200, 0.2, 0), (6000, 400, 0.2, 1), (800, 800, 0.1, 2)])
def test_row_column_pruning_then_compaction_on_the_device(M, N, p, seed):
    """The paper's step (b) on one matrix, device end to end: a row pruning iteration and a column pruning iteration
    with equal ratios (two calls: in one call the column threshold is the one of the matrix as passed in, and after a
    fifth of the rows has gone every column sum of a random matrix lies below it), then the compaction.  The
    dimensions shrink by exactly what the pruning removed, and the compacted matrix is the oracle's compaction of the
    pruned mask."""
    import torch
    rng = np.random.default_rng(300 + seed)
    W = rng.standard_normal((M, N)).astype(np.float32)
    dev = torch.device("cuda:0")
    dW = torch.from_numpy(W).to(dev)
    dm = torch.ones((M, N), dtype=torch.uint8, device=dev)
    rows, none = B.lstm_prune_rows_cols(dW.data_ptr(), dm.data_ptr(), M, N, p, 0.0)
    none2, cols = B.lstm_prune_rows_cols(dW.data_ptr(), dm.data_ptr(), M, N, 0.0, p)
    assert none == 0 and none2 == 0
    assert rows == int(np.ceil(p * M)) and cols == int(np.ceil(p * N))        # no ties in random data: exactly the ratio
    Wp, mp = dW.cpu().numpy(), dm.cpu().numpy()
    got = gpu_compact(Wp, mp, 1)
    ref = ocompact.compact_rows_cols(Wp, mp, 1)
    for g, r in zip(got, ref):
        np.testing.assert_array_equal(g, r)
    assert got[0].size == M - rows and got[1].size == N - cols
    assert got[3].all()                                                       # what is left is dense


@pytest.mark.parametrize("bidir,H,D,T,Bsz,fracs", [
    (False, 96, 40, 9, 1, [0.8, 0.5, 0.65]),      # three layers that shrink by different amounts, batch 1
    (True, 64, 48, 7, 3, [0.75, 0.9]),            # bidirectional: the upper layer reads both directions' kept units
    (False, 1500, 400, 5, 1, [0.798, 0.4173]),    # 1500 -> 1197 in one layer and -> 626 in the other (Sections 5.1, 5.2)
])
def test_layers_pruned_to_different_widths_run_as_one_model(bidir, H, D, T, Bsz, fracs):
    """Row/column pruning leaves every layer its own width.  Each matrix is compacted on the device, the compacted
    matrices make a model with per-layer widths (lstm_create_layers), and its outputs equal the oracle's outputs of
    the full-size pruned model at the kept units."""
    import torch
    layers, ndir = len(fracs), 2 if bidir else 1
    w = inputs.shrink(inputs.c2(Bsz), layers=layers, bidirectional=bidir, input_dim=D, hidden=H, T=T, B=Bsz, keep=0.6,
                      bias="uniform", a=min(0.4, 1.5 / np.sqrt(H)))
    case = inputs.make_case(w, k=6, random_state=True)
    pruned, units, feats = inputs.structure_masks(case, fracs, 0.7925, k=3)
    weights, widths = {}, []
    for l in range(layers):
        for d in range(ndir):
            cur = pruned.weights[(l, d)]
            rx, cx, Wxc, Mxc = gpu_compact(cur["Wx"], cur["Mx"], 4)
            rh, ch, Whc, Mhc = gpu_compact(cur["Wh"], cur["Mh"], 4)
            np.testing.assert_array_equal(rx, units[(l, d)])
            np.testing.assert_array_equal(rh, units[(l, d)])
            np.testing.assert_array_equal(ch, units[(l, d)])
            below = feats if l == 0 else np.concatenate([dd * H + units[(l - 1, dd)] for dd in range(ndir)])
            np.testing.assert_array_equal(cx, below)
            b = np.ascontiguousarray(cur["b"].reshape(4, H)[:, rh].reshape(-1))
            weights[(l, d)] = dict(Wx=Wxc, Mx=Mxc, Wh=Whc, Mh=Mhc, b=b)
        widths.append(len(units[(l, 0)]))
    if H == 1500:
        assert widths == [1197, 626] and len(feats) == 317
    assert len(set(widths)) > 1
    ref_y, ref_h, ref_c = orc.forward_case(pruned)
    last = layers - 1
    ycols = np.concatenate([d * H + units[(last, d)] for d in range(ndir)])
    dev = torch.device("cuda:0")
    m = B.Lstm(layers, len(feats), widths, bidir)
    m.set_weights_from(weights)
    state = lambda s: torch.from_numpy(np.concatenate(
        [s[l * ndir + d][:, units[(l, d)]].ravel() for l in range(layers) for d in range(ndir)])).to(dev)
    y, hT, cT = m.forward(torch.from_numpy(np.ascontiguousarray(pruned.x[:, :, feats])).to(dev), state(pruned.h0),
                          state(pruned.c0))
    desc = B.lstm_describe_plan(m.handle)
    m.close()
    hT, cT = hT.cpu().numpy(), cT.cpu().numpy()
    off = 0
    for l in range(layers):
        for d in range(ndir):
            n, Hc = l * ndir + d, widths[l]
            for name, got, ref in (("hT", hT, ref_h), ("cT", cT, ref_c)):
                g = got[off:off + Bsz * Hc].reshape(Bsz, Hc).astype(np.float64)
                dlt = g - ref[n][:, units[(l, d)]]
                assert np.max(np.abs(dlt)) <= 1e-5, (desc, name, l, d, float(np.max(np.abs(dlt))))
            off += Bsz * Hc
    assert off == hT.size
    dy = y.cpu().numpy().astype(np.float64) - ref_y[:, :, ycols]
    assert np.max(np.abs(dy)) <= 1e-5 and np.linalg.norm(dy) <= 1e-4 * np.linalg.norm(ref_y[:, :, ycols]), desc
