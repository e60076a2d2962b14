"""GPU parity of the H-LSTM cell: liblstm355 (through its C ABI) against the fp64 CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from oracle import hlstm_oracle as horc
from oracle import lstm_oracle as lorc
from paper_1901_10997_amd import binding as B
from paper_1901_10997_amd import inputs
from parity_util import check_case, compare, run_gpu

pytestmark = pytest.mark.gpu

AUTO, DENSE, CSR = B.LSTM_FMT_AUTO, B.LSTM_FMT_DENSE_MASKED, B.LSTM_FMT_ROW_COMPRESSED
PAUTO, STEP, PERSIST = B.LSTM_PLAN_AUTO, B.LSTM_PLAN_STEPWISE, B.LSTM_PLAN_PERSISTENT


def _hw(cid, L, bidir, D, H, G, T, Bn, a=0.4, keep=None, bias="uniform"):
    return inputs.Workload(cid, f"hl_L{L}_D{D}_H{H}_G{G}_T{T}_B{Bn}", L, bidir, D, H, T, Bn, "f32", a, keep, bias, G)


ODD = [
    # L, bidir, D, H, G, T, B, keep
    (1, False, 5, 3, 2, 1, 1, None),
    (1, False, 70, 65, 33, 4, 1, None),
    (2, False, 33, 130, 131, 7, 1, 0.3),
    (1, True, 17, 100, 64, 5, 1, 0.5),
    (2, True, 40, 67, 90, 6, 2, 0.2),
    (1, False, 129, 257, 100, 3, 3, None),
    (3, True, 31, 90, 90, 5, 17, 0.15),
    (1, False, 64, 64, 256, 9, 5, 0.05),
]


@pytest.mark.parametrize("shape", ODD)
@pytest.mark.parametrize("fmt", [DENSE, CSR])
def test_hlstm_odd_shapes_stepwise(shape, fmt):
    L, bidir, D, H, G, T, Bn, keep = shape
    case = inputs.make_case(_hw(80, L, bidir, D, H, G, T, Bn, keep=keep), k=L + H + G, random_state=True)
    desc, _ = check_case(case, fmt, STEP)
    assert ("hlstm-stepwise-pair-csr" if fmt == CSR else "hlstm-stepwise-dense") in desc


@pytest.mark.parametrize("which", ["hidden_layers_empty", "gate_outputs_empty", "input_side_empty", "rows_and_columns_gone", "all_kept_compressed"])
@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, G, T, B
    (2, False, 40, 130, 120, 6, 1),
    (1, True, 33, 72, 80, 5, 3),
])
def test_hlstm_degenerate_masks(which, shape):
    """Masks with nothing kept in one of the three matrices, with whole rows and columns gone, and a mask that keeps
    everything stored in the compressed form; every format and plan against the oracle on the same masks."""
    L, bidir, D, H, G, T, Bn = shape
    case = inputs.make_case(_hw(81, L, bidir, D, H, G, T, Bn, keep=0.3), k=len(which) + G, random_state=True)
    for p in case.weights.values():
        if which == "hidden_layers_empty":
            p["M1x"][:] = 0
            p["M1h"][:] = 0
        if which == "gate_outputs_empty":
            p["M2"][:] = 0
        if which == "input_side_empty":
            p["M1x"][:] = 0
        if which == "rows_and_columns_gone":
            for M in (p["M1x"], p["M1h"], p["M2"]):
                M[::3, :] = 0
                M[:, 1::4] = 0
            p["M2"][0:H, :] = 0            # the forget gate's whole output layer
        if which == "all_kept_compressed":
            for M in (p["M1x"], p["M1h"], p["M2"]):
                M[:] = 1
    for fmt in (DENSE, CSR):
        for plan in (PAUTO, STEP):
            check_case(case, fmt, plan)


def test_poll_pacing_changes_no_bit(monkeypatch):
    """The wait in front of a paced poll (LSTM355_POLL_PACE at lstm_create: units of 64 clocks; default: each kernel's
    measured optimum) only moves the first polling round in time: outputs are bit-identical whatever its length, for the
    batch-1 H-LSTM kernel, for the small-batch recurrence with a device-wide exchange and for the dense fp32 recurrence."""
    cases = [
        (inputs.make_case(_hw(82, 1, False, 40, 300, 280, 12, 1, keep=0.2), k=1, random_state=True), "persist_b1-hlstm"),
        (inputs.make_case(inputs.Workload(82, "wide_b12", 1, False, 64, 1100, 9, 12, "f32", 0.05, 0.1, "uniform"), k=2, random_state=True),
         "persist_batched"),
        (inputs.make_case(inputs.Workload(82, "dense_b8", 1, True, 40, 100, 9, 8, "f32", 0.1, None, "uniform"), k=3, random_state=True),
         "persist-dense-f32"),
    ]
    for case, want in cases:
        outs = []
        for pace in (None, "0", "40"):
            if pace is not None:
                monkeypatch.setenv("LSTM355_POLL_PACE", pace)
            gpu, desc = run_gpu(case, CSR if case.w.keep is not None else DENSE, PAUTO)
            monkeypatch.delenv("LSTM355_POLL_PACE", raising=False)
            assert want in desc, desc
            outs.append(gpu)
        for other in outs[1:]:
            for a, b in zip(outs[0], other):
                assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    check_case(cases[0][0], CSR, PAUTO)
    check_case(cases[1][0], CSR, PAUTO)
    check_case(cases[2][0], DENSE, PAUTO)


def test_hlstm_generic_compressed_kernels_for_long_rows():
    """Rows with more than six 64-entry slices fall back from the paired small-batch kernels to the generic ones."""
    case = inputs.make_case(_hw(80, 1, True, 30, 450, 420, 4, 3, a=0.1), k=9, random_state=True)
    desc, _ = check_case(case, CSR, STEP)
    assert "hlstm-stepwise-csr" in desc


def test_hlstm_handle_kinds_do_not_mix():
    m = B.Lstm(1, 4, 4, gate_hidden=3)
    z = np.zeros((16, 4), np.float32)
    with pytest.raises(B.LstmError) as ei:
        B.lstm_set_weights(m.handle, 0, 0, z, None, z, None, np.zeros(16, np.float32))
    assert ei.value.code == B.LSTM_ERR_STATE
    m.close()
    m = B.Lstm(1, 4, 4)
    with pytest.raises(B.LstmError) as ei:
        B.lstm_set_weights_h(m.handle, 0, 0, np.zeros((12, 4), np.float32), None, np.zeros((12, 4), np.float32), None,
                             np.zeros(12, np.float32), np.zeros((16, 3), np.float32), None, np.zeros(16, np.float32))
    assert ei.value.code == B.LSTM_ERR_STATE
    m.close()
    with pytest.raises(B.LstmError) as ei:
        B.lstm_create_h(1, 4, 4, 3, False, B.LSTM_BF16)
    assert ei.value.code == B.LSTM_ERR_ARG


def test_hlstm_compressed_structure_is_the_mask():
    """The compressed form of all three matrices keeps exactly the mask's positions, in ABI row order."""
    case = inputs.make_case(_hw(81, 1, False, 20, 24, 28, 2, 1, keep=0.3), k=0)
    m = B.Lstm(1, 20, 24, gate_hidden=28)
    m.set_weights_from(case.weights, CSR)
    p = case.weights[(0, 0)]
    for which, wn, mn in ((0, "W1x", "M1x"), (1, "W1h", "M1h"), (2, "W2", "M2")):
        mask = p[mn]
        rp, col, val = B.lstm_get_compressed(m.handle, 0, 0, which, mask.shape[0])
        assert rp[-1] == int(mask.sum()) and len(rp) == mask.shape[0] + 1
        for r in range(mask.shape[0]):
            cols = np.nonzero(mask[r])[0]
            np.testing.assert_array_equal(col[rp[r]:rp[r + 1]], cols)
            np.testing.assert_array_equal(val[rp[r]:rp[r + 1]], p[wn][r, cols])
    m.close()


def test_hlstm_garbage_under_mask_is_invisible_and_runs_are_deterministic():
    case = inputs.make_case(_hw(82, 2, True, 24, 40, 36, 6, 3, keep=0.4), k=1, random_state=True)
    base, _ = run_gpu(case, CSR, STEP)
    again, _ = run_gpu(case, CSR, STEP)
    for a, b in zip(base, again):
        np.testing.assert_array_equal(a, b)
    dirty = {}
    for k, p in case.weights.items():
        q = dict(p)
        for wn, mn in (("W1x", "M1x"), ("W1h", "M1h"), ("W2", "M2")):
            q[wn] = np.where(p[mn] == 1, p[wn], np.float32(np.nan)).astype(np.float32)
        dirty[k] = q
    dcase = inputs.Case(case.w, case.seed, dirty, case.x, case.h0, case.c0)
    for fmt in (CSR, DENSE):
        got, _ = run_gpu(dcase, fmt, STEP)
        ref, _ = run_gpu(case, fmt, STEP)
        for a, b in zip(got, ref):
            assert np.all(np.isfinite(a))
            np.testing.assert_array_equal(a, b)


# ---- batch 1, row-compressed: both products and both exchanges of a step inside one persistent kernel ----------
@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, G, T, keep, cooperative
    (1, False, 40, 150, 150, 11, 0.3, True),
    (1, False, 33, 64, 200, 9, 0.9, True),       # more hidden-layer units than outputs, three slices per row
    (2, False, 90, 200, 70, 8, 0.25, True),      # fewer hidden-layer units than outputs; second layer reads the first
    (1, True, 50, 130, 90, 7, 0.5, False),       # both directions, ordinary launch
    (3, True, 31, 96, 96, 5, 0.15, True),
    (1, False, 20, 333, 257, 1, 0.4, True),      # T = 1: no exchange of h at all
    (1, False, 700, 64, 64, 6, 0.2, True),       # input wider than two elements per thread
    (1, False, 100, 1500, 1500, 3, 0.25, False), # the language-model cell with a quarter kept: six to seven slices per row
    (1, False, 64, 600, 400, 4, 0.6, True),      # six slices
])
def test_hlstm_persistent_batch1(shape):
    L, bidir, D, H, G, T, keep, coop = shape
    case = inputs.make_case(_hw(83, L, bidir, D, H, G, T, 1, a=0.4 if H < 1000 else 0.04, keep=keep), k=H + G + T, random_state=True)
    desc, _ = check_case(case, CSR, PERSIST, cooperative=coop)
    assert "persist_b1-hlstm" in desc
    desc, _ = check_case(case, CSR, STEP)
    assert "hlstm-stepwise" in desc


def test_hlstm_persistent_long_sequence_and_state_chaining():
    case = inputs.make_case(_hw(84, 1, False, 48, 300, 300, 1200, 1, a=0.3, keep=0.15), k=0, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    assert "persist_b1-hlstm" in desc
    # two halves chained through (hT, cT) on one handle equal one run over the whole sequence
    import torch
    full, _, model = run_gpu(case, CSR, PAUTO, return_model=True)
    dev = torch.device("cuda:0")
    x = torch.from_numpy(case.x).to(dev)
    h0 = torch.from_numpy(case.h0).to(dev); c0 = torch.from_numpy(case.c0).to(dev)
    y1, h1, c1 = model.forward(x[:500].contiguous(), h0, c0)
    y2, h2, c2 = model.forward(x[500:].contiguous(), h1, c1)
    model.close()
    np.testing.assert_array_equal(torch.cat([y1, y2]).cpu().numpy(), full[0])
    np.testing.assert_array_equal(h2.cpu().numpy(), full[1])
    np.testing.assert_array_equal(c2.cpu().numpy(), full[2])


@pytest.mark.parametrize("L,bidir", [(1, False), (2, True)])
def test_hlstm_batch1_consecutive_forwards_of_any_length_on_one_handle(L, bidir):
    """The hidden-layer activations of the batch-1 kernel are stamped with one bit (the parity of the steps their array
    has seen), which runs on from one forward to the next: sequences of odd and even lengths in any order on one
    handle, each compared with the oracle, and every one twice in a row (bit-identical)."""
    import torch
    from oracle import hlstm_oracle as horc
    from parity_util import compare
    dev = torch.device("cuda:0")
    base = inputs.make_case(_hw(86, L, bidir, 30, 140, 110, 9, 1, keep=0.3), k=L, random_state=True)
    model = B.Lstm(L, 30, 140, bidir, B.LSTM_F32, gate_hidden=110)
    model.set_weights_from(base.weights, CSR)
    h0 = torch.from_numpy(base.h0).to(dev); c0 = torch.from_numpy(base.c0).to(dev)
    for T in (1, 1, 3, 2, 5, 1, 4, 9, 7, 7, 2):
        import dataclasses
        case = dataclasses.replace(base, w=inputs.shrink(base.w, T=T), x=base.x[:T].copy())
        x = torch.from_numpy(case.x).to(dev)
        first = [t.cpu().numpy() for t in model.forward(x, h0, c0)]
        assert "persist_b1-hlstm" in B.lstm_describe_plan(model.handle)
        again = [t.cpu().numpy() for t in model.forward(x, h0, c0)]
        for a, b in zip(first, again):
            np.testing.assert_array_equal(a, b)
        compare(first, horc.forward_case(case), "f32", f"T={T}")
    model.close()


# ---- small batches, row-compressed: one persistent launch per layer, 2-D grid of unit groups x batch groups -------
@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, G, T, B, keep, cooperative
    (1, False, 40, 150, 150, 11, 2, 0.3, True),
    (1, False, 33, 64, 200, 9, 3, 0.9, True),       # more hidden-layer units than outputs; ragged batch group
    (2, False, 90, 200, 70, 8, 5, 0.25, True),      # fewer hidden-layer units than outputs; two layers share the slots
    (1, True, 50, 130, 90, 7, 16, 0.5, False),      # both directions in one grid, ordinary launch
    (3, True, 31, 96, 96, 5, 17, 0.15, True),
    (1, False, 20, 333, 257, 1, 4, 0.4, True),      # T = 1: no exchange of h at all
    (1, True, 64, 400, 400, 6, 16, 0.35, True),     # three slices per row, 4 units per wave and 4 columns
    (1, False, 30, 37, 41, 9, 33, 0.6, True),       # many batch groups, few units
    (1, False, 400, 1500, 1500, 4, 20, 0.10, False),  # the language-model cell at batch 20: 96 KB of hidden activations
    (1, False, 100, 1100, 1300, 3, 12, 0.10, True),   # per batch group in LDS (offsets beyond 64 KB)
    (2, True, 100, 1200, 1200, 3, 24, 0.10, False),   # two directions that do not fit one grid together: two launches
    (1, False, 100, 1500, 1500, 3, 33, 0.10, True),   # more batch groups than fit the device: runs of batch columns
    (1, True, 80, 800, 800, 3, 64, 0.20, False),
    (1, True, 64, 800, 800, 3, 16, 0.40, False),      # rows of 320 kept entries and more: 22 to 24 slots, two units per wave
    (2, False, 64, 500, 640, 3, 6, 0.33, True),
])
def test_hlstm_persistent_small_batch(shape):
    L, bidir, D, H, G, T, Bn, keep, coop = shape
    case = inputs.make_case(_hw(85, L, bidir, D, H, G, T, Bn, keep=keep), k=H + G + T + Bn, random_state=True)
    desc, _ = check_case(case, CSR, PERSIST, cooperative=coop)
    assert desc.count("persist_batched-hlstm") == L * (2 if bidir else 1)
    desc, _ = check_case(case, CSR, PAUTO, cooperative=coop)
    assert desc.count("persist_batched-hlstm") == L * (2 if bidir else 1)


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, G, T, B, keep
    (1, True, 100, 400, 400, 7, 4, 0.12),
    (2, False, 120, 410, 380, 6, 7, 0.27),
    (1, False, 64, 600, 520, 5, 16, 0.18),
])
def test_hlstm_persistent_small_batch_rows_longer_than_the_slots(shape):
    """A few rows of the recurrent hidden-layer matrix and of the gate-output matrix a few entries longer than all
    others: the slot count follows the common row length and the waves that own those rows add the rest one entry
    at a time."""
    L, bidir, D, H, G, T, Bn, keep = shape
    case = inputs.make_case(_hw(87, L, bidir, D, H, G, T, Bn, keep=keep), k=L, random_state=True)

    def level(M, rows_long, extra):
        n_rows, n_cols = M.shape
        units = n_rows // 4
        target = 32 * max(1, int(round(keep * n_cols / 32.0)))
        for r in range(n_rows):
            on = np.flatnonzero(M[r])
            off = np.flatnonzero(M[r] == 0)
            want = target + (extra if ((r % units) * 4 + r // units) in rows_long else 0)   # ABI row q*units + j is packed row 4j + q
            if len(on) > want:
                M[r, on[want:]] = 0
            elif len(on) < want:
                M[r, off[:want - len(on)]] = 1

    for (l, d), p in case.weights.items():
        level(p["M1h"], (1, 2, 4 * G - 3), 2)      # two long rows in unit 0, one in the last unit
        level(p["M2"], (6, 4 * (H // 2) + 3), 3)
    desc, _ = check_case(case, CSR, PERSIST)
    assert "persist_batched-hlstm-csr+ovf" in desc


def test_hlstm_persistent_small_batch_long_sequence_and_state_chaining():
    case = inputs.make_case(_hw(86, 1, True, 48, 200, 160, 700, 6, a=0.3, keep=0.2), k=0, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    assert "persist_batched-hlstm" in desc
    import torch
    full, _, model = run_gpu(case, CSR, PAUTO, return_model=True)
    dev = torch.device("cuda:0")
    x = torch.from_numpy(case.x).to(dev)
    h0 = torch.from_numpy(case.h0).to(dev); c0 = torch.from_numpy(case.c0).to(dev)
    # repeated forwards on one handle give the same bits (slots and flags restart cleanly)
    ya, ha, ca = model.forward(x, h0, c0)
    yb, hb, cb = model.forward(x, h0, c0)
    model.close()
    np.testing.assert_array_equal(ya.cpu().numpy(), full[0])
    np.testing.assert_array_equal(yb.cpu().numpy(), full[0])
    np.testing.assert_array_equal(hb.cpu().numpy(), full[1])
    np.testing.assert_array_equal(cb.cpu().numpy(), full[2])


@pytest.mark.parametrize("gate_hidden", [0, 170])
def test_one_handle_alternating_batch_sizes(gate_hidden):
    """One handle and one (reused) workspace serve forwards of different batch sizes in turn: the exchange slots, flags
    and activation buffers move inside the workspace with the batch size and must not see each other's leftovers."""
    mk = _hw(88, 2, True, 48, 160, gate_hidden, 9, 6, keep=0.3) if gate_hidden else \
        inputs.Workload(88, "alt_lstm", 2, True, 48, 160, 9, 6, "f32", 0.3, 0.3, "uniform")
    big = inputs.make_case(mk, k=1, random_state=True)
    small = inputs.select_batch(big, [4, 0, 5])
    oracle = horc.forward_case if gate_hidden else lorc.forward_case
    model = None
    try:
        for case in (big, small, big, small):
            out, desc, model = run_gpu(case, CSR, PAUTO, model=model, return_model=True)
            assert "persist_batched" in desc
            compare(out, oracle(case), "f32", f"alternating B={case.w.B}")
    finally:
        if model is not None:
            model.close()


def _random_small_batch_shapes(seed, n, hlstm):
    rng = np.random.Generator(np.random.PCG64(seed))
    shapes = []
    for _ in range(n):
        H = int(rng.integers(40, 640))
        G = int(rng.integers(40, 640)) if hlstm else 0
        D = int(rng.integers(8, 200))
        Bn = int(rng.integers(2, 40))
        # kept entries per row between a few and about 250: one to four 64-entry slices
        K = max(H, G) if hlstm else H
        keep = float(min(0.95, max(0.02, rng.uniform(10, 250) / K)))
        shapes.append((int(rng.integers(1, 3)), bool(rng.integers(0, 2)), D, H, G, int(rng.integers(2, 7)), Bn, round(keep, 3)))
    return shapes


@pytest.mark.parametrize("shape", _random_small_batch_shapes(2024, 12, True) + _random_small_batch_shapes(2025, 12, False))
def test_small_batch_persistent_random_shapes(shape):
    """Seeded random shapes over the (slices per row, units per wave, batch columns) choices of the small-batch kernels."""
    L, bidir, D, H, G, T, Bn, keep = shape
    # weight range tied to the kept fan-in, so that pre-activations stay of order one as in a trained model (the absolute
    # tolerance is stated for that regime)
    a = min(0.4, 1.5 / float(np.sqrt(keep * max(H, G))))
    w = _hw(89, L, bidir, D, H, G, T, Bn, a=a, keep=keep) if G else \
        inputs.Workload(89, f"rnd_L{L}_D{D}_H{H}_T{T}_B{Bn}", L, bidir, D, H, T, Bn, "f32", a, keep, "uniform")
    case = inputs.make_case(w, k=H + Bn, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    print(f"[random-shape] {shape} -> {desc}", flush=True)


@pytest.mark.parametrize("shape", _random_small_batch_shapes(2024, 12, True)[::4] + _random_small_batch_shapes(2025, 12, False)[::3])
def test_random_shapes_with_a_fixed_weight_range(shape):
    """The same shapes with the weight range NOT tied to the fan-in (a = 0.4 throughout): small shapes run with
    pre-activations well below one, large ones with saturated gates.  The tolerance is the usual one; the measured error
    is printed."""
    L, bidir, D, H, G, T, Bn, keep = shape
    w = _hw(91, L, bidir, D, H, G, T, Bn, a=0.4, keep=keep) if G else \
        inputs.Workload(91, f"rndfix_L{L}_D{D}_H{H}_T{T}_B{Bn}", L, bidir, D, H, T, Bn, "f32", 0.4, keep, "uniform")
    case = inputs.make_case(w, k=H + Bn, random_state=True)
    desc, err = check_case(case, CSR, PAUTO)
    print(f"[random-shape, a=0.4] {shape} -> {desc} {err}", flush=True)


def _random_batch1_shapes(seed, n, kind):
    rng = np.random.Generator(np.random.PCG64(seed))
    shapes = []
    for _ in range(n):
        H = int(rng.integers(30, 1400))
        G = int(rng.integers(30, 1400)) if kind == "hlstm" else 0
        D = int(rng.integers(8, 1400))
        K = max(H, G, D)
        keep = None if kind == "dense" else round(float(min(0.95, max(0.02, rng.uniform(10, 400) / K))), 3)
        shapes.append((int(rng.integers(1, 4)), bool(rng.integers(0, 2)), D, H, G, int(rng.integers(1, 8)), keep))
    return shapes


@pytest.mark.parametrize("shape", _random_batch1_shapes(2026, 10, "hlstm") + _random_batch1_shapes(2027, 14, "csr") +
                         _random_batch1_shapes(2028, 8, "dense"))
def test_batch1_random_shapes(shape):
    """Seeded random shapes over the register tiers and slice counts of the batch-1 kernels (dense, row-compressed with
    and without the two-layer wavefront, H-LSTM)."""
    L, bidir, D, H, G, T, keep = shape
    fan = (keep if keep is not None else 1.0) * max(H, G, D)
    a = min(0.4, 1.5 / float(np.sqrt(fan)))
    w = _hw(90, L, bidir, D, H, G, T, 1, a=a, keep=keep) if G else \
        inputs.Workload(90, f"rnd1_L{L}_D{D}_H{H}_T{T}", L, bidir, D, H, T, 1, "f32", a, keep, "uniform")
    case = inputs.make_case(w, k=H + T, random_state=True)
    desc, _ = check_case(case, DENSE if keep is None else CSR, PAUTO)
    print(f"[random-shape] {shape} -> {desc}", flush=True)


def test_hlstm_full_size_language_model():
    """The paper's language-model H-LSTM shape (one layer, 1500 / 1500, embeddings of 400), batch 1, 10 % kept."""
    case = inputs.make_case(inputs.h1(), 0)
    desc, _ = check_case(case, AUTO, PAUTO, cooperative=False)
    assert "persist_b1-hlstm" in desc


@pytest.mark.slow
def test_hlstm_full_size_speech_sampled_columns():
    """The paper's speech H-LSTM shape (3 bidirectional layers, 800 / 800, batch 16); the oracle runs two of the
    sixteen sequences (sequences are independent)."""
    case = inputs.make_case(inputs.h2(), 0)
    desc, _ = check_case(case, AUTO, PAUTO, oracle_cols=[3, 12])
    assert "persist_batched-hlstm" in desc


def test_hlstm_auto_format_compresses_up_to_half_kept():
    """LSTM_FMT_AUTO on an H-LSTM: masks that keep 35 % are held row-compressed (the H-LSTM's dense kernels are the slow
    ones) and the layer runs in the persistent small-batch kernel; unmasked weights stay dense."""
    w = _hw(86, 1, True, 48, 320, 320, 4, 8, keep=0.35)
    desc, _ = check_case(inputs.make_case(w, 3), B.LSTM_FMT_AUTO, PAUTO)
    assert desc.count("persist_batched-hlstm-csr") == 2, desc
    desc, _ = check_case(inputs.make_case(_hw(86, 1, False, 48, 96, 96, 3, 4), 3), B.LSTM_FMT_AUTO, PAUTO)
    assert "dense" in desc.split("rec=")[1], desc

