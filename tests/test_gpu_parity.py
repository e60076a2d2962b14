"""GPU parity: liblstm355 (through its C ABI) against the fp64 CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from oracle import compress as ocomp
from oracle import lstm_oracle as orc
from paper_1901_10997_amd import binding as B
from paper_1901_10997_amd import inputs
from parity_util import check_case, compare, run_gpu

pytestmark = pytest.mark.gpu

AUTO, DENSE, CSR = B.LSTM_FMT_AUTO, B.LSTM_FMT_DENSE_MASKED, B.LSTM_FMT_ROW_COMPRESSED
PAUTO, STEP, PERSIST = B.LSTM_PLAN_AUTO, B.LSTM_PLAN_STEPWISE, B.LSTM_PLAN_PERSISTENT


def _wl(cid, L, bidir, D, H, T, Bn, dtype="f32", a=0.3, keep=None, bias="uniform"):
    return inputs.Workload(cid, f"odd_L{L}_D{D}_H{H}_T{T}_B{Bn}", L, bidir, D, H, T, Bn, dtype, a, keep, bias)


# ---- small odd shapes: tails in every dimension, every plan and format -----------------------------------
ODD = [
    # L, bidir, D, H, T, B, keep
    (1, False, 5, 3, 1, 1, None),
    (1, False, 70, 65, 4, 1, None),
    (2, False, 33, 130, 7, 1, 0.3),
    (1, True, 17, 100, 5, 1, 0.5),
    (2, True, 40, 67, 6, 2, 0.2),
    (1, False, 129, 257, 3, 3, None),
    (3, True, 31, 90, 5, 17, 0.15),
    (1, False, 64, 64, 9, 5, 0.05),
]


@pytest.mark.parametrize("shape", ODD)
@pytest.mark.parametrize("fmt", [DENSE, CSR])
@pytest.mark.parametrize("plan", [PAUTO, STEP])
def test_odd_shapes(shape, fmt, plan):
    L, bidir, D, H, T, Bn, keep = shape
    case = inputs.make_case(_wl(90, L, bidir, D, H, T, Bn, keep=keep), k=L + H, random_state=True)
    check_case(case, fmt, plan)


@pytest.mark.parametrize("waves", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("fmt", [DENSE, CSR])
def test_persistent_group_sizes(waves, fmt):
    case = inputs.make_case(_wl(91, 1, False, 50, 333, 12, 1, keep=0.4), k=waves, random_state=True)
    desc, _ = check_case(case, fmt, PERSIST, waves)
    assert "persist_b1" in desc


@pytest.mark.parametrize("L", [2, 3, 4])
@pytest.mark.parametrize("H,D,keep", [(150, 90, 0.3), (64, 200, 0.9), (700, 300, 0.05)])
def test_layer_wavefront_stacks(L, H, D, keep):
    """Unidirectional row-compressed stacks at batch 1 run two layers per launch (diagonal wavefront)."""
    case = inputs.make_case(_wl(99, L, False, D, H, 11, 1, keep=keep), k=L, random_state=True)
    desc, _ = check_case(case, CSR, PERSIST)
    assert "wavefront" in desc
    check_case(inputs.make_case(_wl(99, L, False, D, H, 1, 1, keep=keep), k=L), CSR, PERSIST)   # T = 1


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, keep -- a few rows a little longer than a multiple of 64 kept entries: the batch-1 kernel holds
    # the common row length in registers and takes the remainder from per-unit overflow lists
    (1, False, 400, 400, 0.12),
    (2, False, 400, 400, 0.12),
    (1, True, 300, 520, 0.10),
    (3, False, 410, 410, 0.27),
    (2, False, 900, 600, 0.18),
])
def test_batch1_overflow_rows(shape):
    L, bidir, D, H, keep = shape
    case = inputs.make_case(_wl(98, L, bidir, D, H, 9, 1, keep=keep), k=L, random_state=True)
    desc, _ = check_case(case, CSR, PERSIST)
    assert "+ovf" in desc
    check_case(case, CSR, PERSIST, 4)   # another workgroup size


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, T, B, keep  -- small-batch row-compressed stacks: time loop on the device
    (2, True, 64, 200, 9, 16, 0.15),
    (1, False, 40, 333, 7, 20, 0.10),
    (2, False, 48, 130, 6, 3, 0.5),
    (1, True, 32, 96, 5, 33, 0.3),
    (2, True, 200, 1500, 4, 20, 0.10),   # two directions that do not fit one grid together: the layer is cut in two launches
    (2, False, 100, 1500, 3, 45, 0.10),  # more batch groups than fit the device: runs of batch columns, a launch each
    (1, True, 64, 2048, 3, 21, 0.08),    # both cuts, runs of unequal length
    (1, False, 100, 1500, 3, 17, 0.15),  # rows of 225 kept entries and more: 16 to 18 slots
    (1, True, 64, 1500, 3, 16, 0.20),    # 300 and more: 20 to 22 slots, four units and four columns at the register limit
    (2, False, 64, 2048, 2, 8, 0.15),    # 310 and more: 22 to 24 slots
])
def test_small_batch_persistent(shape):
    L, bidir, D, H, T, Bn, keep = shape
    a = 0.3 if H < 1000 else 0.04
    case = inputs.make_case(_wl(88, L, bidir, D, H, T, Bn, a=a, keep=keep), k=H + Bn, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    assert desc.count("persist_batched") == L * (2 if bidir else 1)
    desc, _ = check_case(case, CSR, STEP)
    assert "stepwise" in desc


def test_auto_format_keeps_both_directions_of_a_layer_in_one_form():
    """Masks that keep a quarter of the entries sit on the threshold of LSTM_FMT_AUTO: the two directions of a layer
    must not end up in different forms (the time-loop kernels take both directions only in one form)."""
    for seed in range(5):
        case = inputs.make_case(_wl(96, 2, True, 48, 256, 4, 8, keep=0.25), seed)
        desc, _ = check_case(case, AUTO, PAUTO)
        assert "stepwise" not in desc, desc


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, T, B, keep -- recurrent rows a little longer than a multiple of 64 kept entries (slot counts 6,
    # 8 and 10 of the quarter-wave form, with entries whose bank is full placed by the packer's second pass)
    (2, True, 100, 400, 7, 6, 0.12),
    (1, False, 120, 600, 5, 20, 0.18),
    (1, False, 64, 410, 6, 3, 0.27),
])
def test_small_batch_persistent_overflow_rows(shape):
    L, bidir, D, H, T, Bn, keep = shape
    case = inputs.make_case(_wl(89, L, bidir, D, H, T, Bn, keep=keep), k=H + Bn, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    assert "persist_batched-q16" in desc


@pytest.mark.parametrize("shape", [
    # bidir, D, H, T, B, keep, long rows (packed row = 4 * unit + gate), extra entries per long row
    (False, 48, 256, 6, 5, 0.2, (0, 1, 402, 1023), 2),       # two long rows in one unit, one in the last unit
    (True, 40, 300, 5, 12, 0.15, (7, 600, 601, 1198), 2),
    (False, 32, 520, 4, 3, 0.1, (5, 2079), 4),                # the most a unit may hold outside the slots
])
def test_small_batch_persistent_rows_longer_than_the_slots(shape):
    """A handful of recurrent rows a few entries longer than all others: the slot count follows the common row
    length and those entries are added one at a time by the waves that own them."""
    bidir, D, H, T, Bn, keep, rows, extra = shape
    case = inputs.make_case(_wl(97, 1, bidir, D, H, T, Bn, keep=keep), k=H + Bn, random_state=True)
    for (l, d), p in case.weights.items():
        Mh = p["Mh"]
        # every row to the same length (a multiple of 32: the slots are then exactly full), the chosen rows longer
        target = 32 * max(1, int(round(keep * H / 32.0)))
        for r in range(4 * H):
            on = np.flatnonzero(Mh[r])
            off = np.flatnonzero(Mh[r] == 0)
            want = target + (extra if ((r % H) * 4 + r // H) in rows else 0)   # ABI row q*H + j is packed row 4j + q
            if len(on) > want:
                Mh[r, on[want:]] = 0
            elif len(on) < want:
                Mh[r, off[:want - len(on)]] = 1
    desc, _ = check_case(case, CSR, PAUTO)
    assert "persist_batched-q16+ovf" in desc


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, T, B, keep -- row-compressed input matrices, at least 64 input rows, few kept weights: the
    # projection runs over the kept entries only (ragged last tile of four input rows, widths that are no multiple of
    # four, the widest input the kernel takes, both directions in one launch, a second layer fed by two directions)
    (1, True, 333, 200, 9, 11, 0.10),
    (2, False, 2048, 96, 4, 17, 0.08),
    (1, False, 1601, 300, 5, 13, 0.12),
    (2, True, 90, 260, 7, 10, 0.15),
])
def test_projection_over_kept_entries(shape):
    L, bidir, D, H, T, Bn, keep = shape
    case = inputs.make_case(_wl(96, L, bidir, D, H, T, Bn, keep=keep), k=H + Bn, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    assert "proj=q16" in desc


def test_projection_over_kept_entries_rows_longer_than_the_slots():
    """Input-side rows a few entries longer than all others: the slot count follows the common row length and the
    waves that own those rows add the remaining entries one at a time."""
    D, H, T, Bn = 512, 128, 6, 12
    case = inputs.make_case(_wl(95, 1, True, D, H, T, Bn, keep=0.1), k=3, random_state=True)
    for (l, d), p in case.weights.items():
        Mx = p["Mx"]
        for r in range(4 * H):
            on = np.flatnonzero(Mx[r])
            off = np.flatnonzero(Mx[r] == 0)
            want = 64 + (3 if r in (0, H, 2 * H + 77, 4 * H - 1) else 0)   # 64 entries = four full slots
            if len(on) > want:
                Mx[r, on[want:]] = 0
            elif len(on) < want:
                Mx[r, off[:want - len(on)]] = 1
    desc, _ = check_case(case, CSR, PAUTO)
    assert "proj=q16" in desc


def test_bf16_small():
    for Bn, keep in ((1, None), (3, 0.3), (9, None)):
        case = inputs.make_case(_wl(92, 2, False, 48, 96, 6, Bn, dtype="bf16", a=0.2, keep=keep), k=Bn, random_state=True)
        for fmt in (DENSE, CSR):
            check_case(case, fmt, PAUTO)


@pytest.mark.parametrize("Bn", [32, 40, 130])
@pytest.mark.parametrize("plan", [PAUTO, STEP])
def test_bf16_matrix_core_recurrence(Bn, plan):
    """bf16 dense stacks at batch >= 32 run the recurrence on the matrix cores (batch tail included): with the time
    loop on the device when H % 128 == 0, H <= 1024 and the tiles fit one per compute unit, else (or when the
    stepwise plan is forced) with one launch per step (H % 256 == 0)."""
    case = inputs.make_case(_wl(89, 2, False, 64, 256, 5, Bn, dtype="bf16", a=0.1), k=Bn, random_state=True)
    desc, _ = check_case(case, DENSE, plan)
    assert ("persist-mfma" if plan == PAUTO else "stepwise-mfma") in desc


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, T, B, random initial state, cooperative launch
    (1, False, 64, 128, 1, 64, False, True),     # one step, no exchange at all
    (2, False, 96, 384, 9, 70, True, True),      # three k16 steps per wave, batch tail
    (1, True, 64, 256, 7, 100, True, True),      # both directions (one launch each)
    (2, False, 64, 512, 12, 33, False, False),   # zero initial state, ordinary launch
    (1, False, 128, 1024, 6, 64, True, False),   # widest supported hidden size: 64 tiles along the gate rows
])
def test_bf16_persistent_matrix_core_shapes(shape):
    L, bidir, D, H, T, Bn, rs, coop = shape
    case = inputs.make_case(_wl(86, L, bidir, D, H, T, Bn, dtype="bf16", a=0.08), k=H + T, random_state=rs)
    desc, _ = check_case(case, DENSE, PAUTO, cooperative=coop)
    assert "persist-mfma" in desc


def _random_bf16_shapes(seed, n):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(n):
        H = 128 * int(rng.integers(1, 9))
        out.append((int(rng.integers(1, 3)), bool(rng.integers(0, 2)), 8 * int(rng.integers(2, 40)), H,
                    int(rng.integers(2, 8)), int(rng.integers(32, 300))))
    return out


@pytest.mark.parametrize("shape", _random_bf16_shapes(2029, 8))
def test_bf16_persistent_matrix_core_random_shapes(shape):
    """Seeded random batch sizes (ragged 32-row tiles) and hidden widths over the bf16 persistent recurrence."""
    L, bidir, D, H, T, Bn = shape
    if ((Bn + 31) // 32) * (H // 32) > 256:
        pytest.skip("more tiles than compute units: served by the stepwise kernel, covered elsewhere")
    case = inputs.make_case(_wl(87, L, bidir, D, H, T, Bn, dtype="bf16", a=min(0.08, 1.5 / float(np.sqrt(H)))), k=H + Bn,
                            random_state=True)
    desc, _ = check_case(case, DENSE, PAUTO)
    assert "persist-mfma" in desc


def test_bf16_persistent_matrix_core_long_sequence():
    """Many steps: the flag tags keep growing across steps and across the two layers' launches."""
    case = inputs.make_case(_wl(85, 2, False, 64, 256, 400, 64, dtype="bf16", a=0.06), k=1, random_state=True)
    desc, _ = check_case(case, DENSE, PAUTO)
    assert "persist-mfma" in desc


def test_bf16_persistent_full_size_many_forwards_back_to_back():
    """The throughput configuration, 60 forwards issued without a synchronisation in between (15 000 exchange rounds of
    256 tiles): a tile that has seen every flag of a step may raise its own flag to the next tag before a slower tile
    has looked, so the pollers must accept "at least" the tag they wait for.  No bounded wait may expire, and every
    forward gives the same bits."""
    import torch
    case = inputs.make_case(inputs.c5(), 0)
    first, desc, model = run_gpu(case, cooperative=False, return_model=True)
    assert "persist-mfma" in desc
    dev = torch.device("cuda:0")
    x = torch.from_numpy(case.x).to(dev).to(torch.bfloat16)
    outs = None
    for _ in range(60):
        outs = model.forward(x, check=False)
    torch.cuda.synchronize()
    B.lstm_check(model.handle)
    for a, b in zip(first, outs):
        assert np.array_equal(a, b.cpu().numpy())
    model.close()


@pytest.mark.parametrize("name", ["c1", "c4", "h2"])
def test_full_size_forwards_back_to_back_give_the_same_bits(name):
    """The workloads whose exchange goes through one XCD's L2, 20 forwards issued without a synchronisation in between:
    no bounded wait expires and every forward reproduces the first one bit for bit (a hand-over that let a flag or a
    tag overtake its data would show up as a difference)."""
    import torch
    case = inputs.make_case({"c1": inputs.c1, "c4": inputs.c4, "h2": inputs.h2}[name](), 0)
    first, desc, model = run_gpu(case, cooperative=False, return_model=True)
    assert "persist" in desc
    x = torch.from_numpy(case.x).to(torch.device("cuda:0"))
    outs = None
    for _ in range(20):
        outs = model.forward(x, check=False)
    torch.cuda.synchronize()
    B.lstm_check(model.handle)
    for a, b in zip(first, outs):
        assert np.array_equal(a, b.cpu().numpy())
    model.close()


@pytest.mark.parametrize("D", [192, 96, 320])
def test_bf16_large_projection_ragged_tiles(D):
    """bf16 projections with T*B >= 2048 rows and 4H >= 512 columns take the 256 x 256 persistent-tile kernel
    (64-wide K slabs when D % 64 == 0, 32-wide otherwise); 2100 rows and 544 columns leave partial tiles on
    both axes, and more tiles than one pass over the device's compute units is not needed for that."""
    case = inputs.make_case(_wl(87, 1, False, D, 136, 7, 300, dtype="bf16", a=0.1), k=D, random_state=True)
    check_case(case, DENSE, PAUTO)


def test_empty_sequences_are_noops():
    m = B.Lstm(1, 4, 4)
    case = inputs.make_case(_wl(93, 1, False, 4, 4, 2, 1), 0)
    m.set_weights_from(case.weights)
    B.lstm_forward(m.handle, 0, 1, None, None, None, None, None, None, None, 0, None)
    B.lstm_forward(m.handle, 3, 0, None, None, None, None, None, None, None, 0, None)
    m.close()


def test_error_paths_with_a_device():
    import torch
    m = B.Lstm(2, 4, 4)
    case = inputs.make_case(_wl(94, 2, False, 4, 4, 2, 1), 0)
    x = torch.zeros((2, 1, 4), device="cuda:0")
    with pytest.raises(B.LstmError) as ei:      # no weights yet
        m.forward(x)
    assert ei.value.code == B.LSTM_ERR_STATE
    p = case.weights[(0, 0)]
    B.lstm_set_weights(m.handle, 0, 0, p["Wx"], None, p["Wh"], None, p["b"])
    with pytest.raises(B.LstmError) as ei:      # layer 1 still missing
        m.forward(x)
    assert ei.value.code == B.LSTM_ERR_STATE
    with pytest.raises(B.LstmError) as ei:
        B.lstm_set_weights(m.handle, 2, 0, p["Wx"], None, p["Wh"], None, p["b"])
    assert ei.value.code == B.LSTM_ERR_SHAPE
    bad = np.full(p["Wh"].shape, 2, np.uint8)
    with pytest.raises(B.LstmError) as ei:
        B.lstm_set_weights(m.handle, 0, 0, p["Wx"], None, p["Wh"], bad, p["b"])
    assert ei.value.code == B.LSTM_ERR_ARG
    m.set_weights_from(case.weights)
    y = torch.empty((2, 1, 4), device="cuda:0")
    ws = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(B.LstmError) as ei:      # workspace too small
        B.lstm_forward(m.handle, 2, 1, x.data_ptr(), None, None, y.data_ptr(), None, None, ws.data_ptr(), 16, None)
    assert ei.value.code == B.LSTM_ERR_NOMEM
    m.close()


# ---- mask and index handling: bit-exact ---------------------------------------------------------------------
def test_compressed_structure_is_the_mask_bit_exact():
    case = inputs.make_case(_wl(95, 2, True, 37, 29, 3, 1, keep=0.2), 0)
    # plant kept zeros and negative zeros: they stay stored entries
    p = case.weights[(1, 1)]
    kept = np.argwhere(p["Mh"] == 1)
    p["Wh"][tuple(kept[0])] = 0.0
    p["Wh"][tuple(kept[1])] = -0.0
    m = B.Lstm(2, 37, 29, True)
    m.set_weights_from(case.weights, CSR)
    for (l, d), q in case.weights.items():
        for which, (wn, mn) in enumerate((("Wx", "Mx"), ("Wh", "Mh"))):
            rp, col, val = B.lstm_get_compressed(m.handle, l, d, which, 4 * 29)
            rp_o, col_o, val_o = ocomp.row_compress(q[wn], q[mn])
            assert np.array_equal(rp, rp_o)
            assert np.array_equal(col, col_o.astype(np.int32))
            assert np.array_equal(val.view(np.uint32), val_o.view(np.uint32))
    m.close()
    # with no mask the structure is every position
    c2 = inputs.make_case(_wl(95, 1, False, 6, 5, 2, 1), 1)
    m = B.Lstm(1, 6, 5)
    m.set_weights_from(c2.weights, CSR)
    rp, col, val = B.lstm_get_compressed(m.handle, 0, 0, 0, 20)
    assert np.array_equal(rp, np.arange(21) * 6) and np.array_equal(col, np.tile(np.arange(6), 20))
    m.close()


@pytest.mark.parametrize("fmt", [DENSE, CSR])
@pytest.mark.parametrize("Bn", [1, 4])
def test_garbage_under_zero_mask_is_bit_invisible_and_runs_are_deterministic(fmt, Bn):
    case = inputs.make_case(_wl(96, 2, False, 45, 70, 6, Bn, keep=0.3), 0, random_state=True)
    out1, _ = run_gpu(case, fmt)
    out2, _ = run_gpu(case, fmt)
    for a, b in zip(out1, out2):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))       # same bits, run to run
    junk = inputs.make_case(_wl(96, 2, False, 45, 70, 6, Bn, keep=0.3), 0, random_state=True)
    for q in junk.weights.values():
        q["Wx"][q["Mx"] == 0] = np.nan
        q["Wh"][q["Mh"] == 0] = np.float32(3e38)
    out3, _ = run_gpu(junk, fmt)
    for a, b in zip(out1, out3):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_state_chaining_matches_one_long_run():
    case = inputs.make_case(_wl(97, 2, False, 20, 77, 10, 1, keep=0.5), 0)
    full, _ = run_gpu(case)
    import dataclasses
    a = dataclasses.replace(case, x=case.x[:4].copy())
    outa, _ = run_gpu(a)
    b = dataclasses.replace(case, x=case.x[4:].copy(), h0=outa[1], c0=outa[2])
    outb, _ = run_gpu(b)
    assert np.array_equal(outa[0], full[0][:4])
    assert np.array_equal(outb[0], full[0][4:]) and np.array_equal(outb[1], full[1]) and np.array_equal(outb[2], full[2])


def test_repeated_forwards_on_one_handle_and_long_sequence():
    """Many launches reuse the exchange slots (tags keep growing); a long sequence stresses the exchange."""
    case = inputs.make_case(_wl(98, 1, False, 16, 96, 2000, 1, a=0.2), 0)
    ref = orc.forward_case(case)
    out, desc, model = run_gpu(case, DENSE, PERSIST, return_model=True)
    compare(out, ref, "f32", "long")
    for _ in range(5):
        out2, _ = run_gpu(case, DENSE, PERSIST, model=model)
        for a, b in zip(out, out2):
            assert np.array_equal(a, b)
    model.close()


@pytest.mark.parametrize("layers,bidir,D,H,T,Bn,keep", [(2, False, 40, 96, 12, 1, 0.3), (1, True, 24, 96, 15, 4, 0.4),
                                                     (1, False, 64, 128, 9, 64, None)])
def test_forward_on_a_side_stream(layers, bidir, D, H, T, Bn, keep):
    """Every kernel and every clearing of exchange state goes to the caller's stream: a forward issued on a stream other
    than the default one (default priority), with nothing ordering it against the default stream, gives the same bits
    as on the default stream - twice, so that the second run starts from the slots the first one left."""
    import torch
    case = inputs.make_case(_wl(96, layers, bidir, D, H, T, Bn, keep=keep), 1, random_state=True)
    ref = orc.forward_case(case)
    base, desc, model = run_gpu(case, return_model=True)
    compare(base, ref, "f32", f"default stream {desc}")
    dev = torch.device("cuda:0")
    x = torch.from_numpy(case.x).to(dev)
    h0, c0 = torch.from_numpy(case.h0).to(dev), torch.from_numpy(case.c0).to(dev)
    torch.cuda.synchronize()
    side = torch.cuda.Stream(device=dev)
    for _ in range(2):
        with torch.cuda.stream(side):
            y, hT, cT = model.forward(x, h0, c0)
        side.synchronize()
        for a, b in zip(base, (y, hT, cT)):
            assert np.array_equal(a, b.cpu().numpy())
    model.close()


def test_long_sequence_small_batch_persistent():
    """1500 steps through the per-batch-group exchange of the small-batch persistent kernel."""
    case = inputs.make_case(_wl(87, 1, True, 24, 96, 1500, 4, a=0.2, keep=0.4), 0)
    desc, _ = check_case(case, CSR, PAUTO)
    assert "persist_batched" in desc


@pytest.mark.parametrize("wl", ["c1", "c2_b1", "c2_b20", "c3_1312"])
def test_ordinary_launch_mode_full_size(wl):
    """The launch configuration the benchmark times: persistent kernels started with an ordinary launch."""
    w = {"c1": inputs.c1(), "c2_b1": inputs.c2(1), "c2_b20": inputs.c2(20), "c3_1312": inputs.c3(1312)}[wl]
    desc, _ = check_case(inputs.make_case(w, 1), AUTO, PAUTO, cooperative=False)
    assert "persist" in desc


# ---- the five configurations at full size ------------------------------------------------------------------
@pytest.mark.parametrize("k", [0, 1, 2])
@pytest.mark.parametrize("plan", [PAUTO, STEP])
def test_c1_full(k, plan):
    check_case(inputs.make_case(inputs.c1(), k), AUTO, plan)


def test_c1_random_state():
    check_case(inputs.make_case(inputs.c1(), 0, random_state=True))


@pytest.mark.parametrize("Bn", [1, 20])
@pytest.mark.parametrize("fmt", [AUTO, DENSE])
def test_c2_full(Bn, fmt):
    for k in ((0, 1, 2) if fmt == AUTO else (0,)):
        check_case(inputs.make_case(inputs.c2(Bn), k), fmt)


def test_c2_random_state():
    check_case(inputs.make_case(inputs.c2(1), 0, random_state=True))
    check_case(inputs.make_case(inputs.c2(20), 0, random_state=True))


@pytest.mark.parametrize("H", inputs.c3_hidden_sizes() + [1284, 1300, 1900])
def test_c3_points(H):
    """Every width of the latency-hysteresis sweep (H = 64..2048 step 32, Section 3) plus three widths off the grid:
    each width selects its own registers-per-row count, workgroup size, fused or separate input projection and
    placement, and each of them is compared with the oracle."""
    desc, _ = check_case(inputs.make_case(inputs.c3(H), 0), cooperative=(H % 64 == 0))
    assert ("proj=fused-dense,rec=persist_b1-dense" if H <= 1280 else "proj=dense,rec=persist_b1-dense") in desc


def test_latency_sweep_entry_point():
    """lstm_latency_sweep itself (Section 3 profile over the gate dimension): positive, ordered percentiles and
    hysteresis flags that equal lstm_find_lhp at margin 0 on the returned medians."""
    Hs = [96, 64, 160]
    med, p10, p90, flags = B.lstm_latency_sweep(Hs, T=6, B=1, warmup=1, iters=3)
    assert np.all(med > 0) and np.all(p10 <= med + 1e-9) and np.all(med <= p90 + 1e-9)
    ref, _ = B.lstm_find_lhp(Hs, med, 0.0)
    np.testing.assert_array_equal(flags, ref)
    assert flags[2] == 1                                   # the largest dimension always is one
    with pytest.raises(B.LstmError):
        B.lstm_latency_sweep(Hs, T=0, B=1, warmup=0, iters=1)
    empty = B.lstm_latency_sweep([], T=6, B=1, warmup=0, iters=1)        # no points: a no-op
    assert all(len(a) == 0 for a in empty)


@pytest.mark.slow
def test_c4_full_sampled_columns():
    for k in (0, 1, 2):
        check_case(inputs.make_case(inputs.c4(), k, random_state=(k == 2)), AUTO, oracle_cols=[0, 9] if k == 0 else [15])


@pytest.mark.slow
def test_c4_full_dense_masked_sampled_columns():
    """The same five bidirectional layers with the weights held dense-masked (what `bench.py --workload c4_dense`
    times): matrix-core fp32 projection and the dense fp32 persistent recurrence at full size."""
    desc, _ = check_case(inputs.make_case(inputs.c4(), 3), DENSE, oracle_cols=[4, 14])
    assert desc.count("rec=persist-dense-f32") == 10


@pytest.mark.slow
def test_c5_full_sampled_columns():
    for k in (0, 1, 2):
        check_case(inputs.make_case(inputs.c5(), k, random_state=(k == 2)), AUTO, oracle_cols=[0, 131, 255] if k == 0 else [77])


def test_model_level_latency_sweep_runs_every_family():
    """lstm_latency_sweep_model: stacked / bidirectional / masked / H-LSTM points all produce a positive latency and
    flags that agree with lstm_find_lhp on the returned curve."""
    Hs = [96, 64, 128]
    for kw in (dict(layers=1), dict(layers=2, bidirectional=True, keep=0.3, B=3, T=6),
               dict(layers=1, gate_hidden=True, keep=0.2, T=5), dict(layers=2, gate_hidden=True, B=2, T=4),
               dict(layers=2, dtype=B.LSTM_BF16, B=40, T=3)):
        args = dict(T=8, B=1, warmup=1, iters=3)
        args.update(kw)
        med, p10, p90, flags = B.lstm_latency_sweep_model(Hs, [48, 32, 200], **args)
        assert np.all(med > 0) and np.all(p10 <= med + 1e-9) and np.all(med <= p90 + 1e-9)
        ref, _ = B.lstm_find_lhp(Hs, med, 0.0)
        np.testing.assert_array_equal(flags, ref)
    with pytest.raises(B.LstmError):
        B.lstm_latency_sweep_model(Hs, None, gate_hidden=True, dtype=B.LSTM_BF16, warmup=0, iters=1)


@pytest.mark.parametrize("n,batch,keep", [(64, 16, 0.5), (260, 16, 0.1), (512, 5, 1.0), (1000, 16, 0.05), (132, 70, 0.3),
                                          (2048, 16, 0.1), (4096, 16, 0.05), (1500, 16, None), (5124, 3, 0.02),
                                          # one to four 16-row tiles of input rows, widths that end inside a tile
                                          (260, 35, 0.5), (516, 64, None), (72, 1, None), (1316, 48, 0.3), (2052, 33, None)])
@pytest.mark.parametrize("fmt", [DENSE, CSR])
def test_standalone_product_against_the_oracle(n, batch, keep, fmt):
    """lstm_bench_matmul on caller-supplied seeded operands (Section 3, matmul latency figures): the product of either
    format equals the fp64 oracle's X (W (x) Msk)^T within the fp32 tolerance; what lies under a zero mask byte is
    invisible to the bits of the result."""
    from oracle import matmul as omm
    X, W, M = inputs.matmul_operands(n, batch, keep, seed=n + batch)
    ref = omm.masked_product(X, W, M)
    _, y = B.lstm_bench_matmul(n, batch, 1.0, fmt, iters=2, want_product=True, X=X, W=W, mask=M)
    d = y.astype(np.float64) - ref
    assert np.max(np.abs(d)) <= 1e-5 and np.linalg.norm(d) / np.linalg.norm(ref) <= 1e-4, (np.max(np.abs(d)),)
    if M is not None:
        Wj = W.copy()
        Wj[M == 0] = np.float32(np.nan)
        _, y2 = B.lstm_bench_matmul(n, batch, 1.0, fmt, iters=1, want_product=True, X=X, W=Wj, mask=M)
        assert np.array_equal(y.view(np.uint32), y2.view(np.uint32))


def test_standalone_product_seeded_operands_and_errors():
    """With no operands given the library draws its own from the seed: both formats then multiply the same ones, the
    seed changes them, and the product has the scale the distributions imply (n * keep * E[w^2] E[x^2] = n keep / 300)."""
    n, batch, keep = 260, 16, 0.1
    _, yd = B.lstm_bench_matmul(n, batch, keep, DENSE, seed=7, iters=2, want_product=True)
    _, yc = B.lstm_bench_matmul(n, batch, keep, CSR, seed=7, iters=2, want_product=True)
    np.testing.assert_allclose(yc, yd, rtol=0, atol=2e-5)
    var = float(np.mean(yd.astype(np.float64) ** 2))
    assert 0.6 * n * keep / 300 < var < 1.6 * n * keep / 300
    _, other = B.lstm_bench_matmul(n, batch, keep, DENSE, seed=8, iters=1, want_product=True)
    assert np.max(np.abs(other - yd)) > 1e-3
    X, W, M = inputs.matmul_operands(64, 4, 0.5, seed=1)
    with pytest.raises(B.LstmError):
        B.lstm_bench_matmul(64, 4, 1.0, DENSE, X=X)                       # W missing
    with pytest.raises(B.LstmError):
        B.lstm_bench_matmul(64, 4, 1.0, DENSE, X=X, W=W, mask=M * 2)      # mask byte not in {0, 1}
    with pytest.raises(B.LstmError):
        B.lstm_bench_matmul(64, 4, 0.0, DENSE)                            # keep outside (0, 1]


def test_expired_waits_are_reported_and_nothing_hangs(monkeypatch):
    """Every wait inside the persistent kernels is bounded.  With the bound forced down to two polls (environment
    variable read at lstm_create) a forward either completes correctly (the values happened to be there) or drains
    and reports LSTM_ERR_TIMEOUT from the check that follows; in both cases it returns, the flag is cleared by the
    check, and a handle created afterwards with the normal bound works."""
    import torch
    families = [
        (_wl(70, 1, False, 40, 300, 40, 1), DENSE, "persist_b1-dense"),
        (_wl(70, 2, False, 60, 500, 40, 1, keep=0.2), CSR, "wavefront"),
        (_wl(70, 1, True, 48, 400, 30, 12, keep=0.15), CSR, "persist_batched"),
        (_wl(70, 1, False, 64, 512, 30, 128, dtype="bf16", a=0.05), DENSE, "persist-mfma"),
        (_wl(70, 1, True, 48, 400, 30, 12), DENSE, "persist-dense-f32"),
        (inputs.Workload(70, "hl", 1, False, 40, 400, 30, 1, "f32", 0.3, 0.2, "uniform", 400), CSR, "persist_b1-hlstm"),
        (inputs.Workload(70, "hlb", 1, True, 40, 300, 20, 6, "f32", 0.3, 0.2, "uniform", 260), CSR, "persist_batched-hlstm"),
    ]
    monkeypatch.setenv("LSTM355_SPIN_LIMIT", "1")
    timeouts = 0
    for w, fmt, want in families:
        case = inputs.make_case(w, 0)
        try:
            gpu, desc = run_gpu(case, fmt, PAUTO)
        except B.LstmError as e:
            assert e.code == B.LSTM_ERR_TIMEOUT
            timeouts += 1
            continue
        assert want in desc
        from oracle import hlstm_oracle as horc
        ref = (horc if w.gate_hidden else orc).forward_case(case)
        compare(gpu, ref, w.dtype, w.name)
    monkeypatch.delenv("LSTM355_SPIN_LIMIT")
    assert timeouts >= 1      # exchanging across the whole device within two polls every step does not happen
    for w, fmt, want in families:
        desc, _ = check_case(inputs.make_case(w, 0), fmt, PAUTO)
        assert want in desc


def test_group_exchange_yardstick_and_the_one_xcd_check():
    """The exchange yardstick inside groups: spread over the XCDs, placed on one XCD each (every group must then pass the
    check made from the hardware's XCD ids), and with workgroup-scope stores on top (what the product kernels do);
    argument errors for shapes that cannot be placed."""
    spread, ver0 = B.lstm_bench_group_exchange(1024, 32, 8, False, False, steps=50, iters=2)
    placed, ver1 = B.lstm_bench_group_exchange(1024, 32, 8, True, False, steps=50, iters=2)
    local, ver2 = B.lstm_bench_group_exchange(1024, 32, 8, True, True, steps=50, iters=2)
    assert ver0 == 0 and ver1 == 8 and ver2 == 8
    assert 0.1 < local < 20 and 0.1 < placed < 20 and 0.1 < spread < 20
    us, ver = B.lstm_bench_group_exchange(70, 3, 5, True, True, steps=20, iters=1)     # padding block ids, ragged shares
    assert ver == 5 and us > 0
    with pytest.raises(B.LstmError):
        B.lstm_bench_group_exchange(3000, 24, 10, True, True)                              # two groups of 24 per XCD
    with pytest.raises(B.LstmError):
        B.lstm_bench_group_exchange(100, 65, 1, False, False)


@pytest.mark.parametrize("name", ["c1", "c4", "c5", "h2", "dense_narrow"])
def test_l2_handover_off_gives_the_same_bits(name, monkeypatch):
    """The workloads whose exchange is handed over through one XCD's L2, run with that hand-over on and with every
    exchange store forced to device scope (LSTM355_L2_HANDOVER=0 at lstm_create): same placement, same arithmetic, so
    the outputs must be bit-identical; a hand-over that delivered a stale value would show as a difference."""
    w = {"c1": inputs.c1, "c4": inputs.c4, "c5": inputs.c5, "h2": inputs.h2,
         "dense_narrow": lambda: _wl(97, 2, True, 64, 256, 40, 16, a=0.1)}[name]()   # dense fp32 at batch, 32 workgroups per group
    if name in ("c4", "h2"):
        w = inputs.shrink(w, T=60)
    case = inputs.make_case(w, 1)
    on, desc_on = run_gpu(case, cooperative=False)
    monkeypatch.setenv("LSTM355_L2_HANDOVER", "0")
    off, desc_off = run_gpu(case, cooperative=False)
    monkeypatch.delenv("LSTM355_L2_HANDOVER")
    assert desc_on == desc_off and "persist" in desc_on
    for a, b in zip(on, off):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, T, dtype -- dense batch-1 layers of at most 128 units on one XCD: every wave polls the slots
    # into its own registers and publishes its own h (no LDS copy, no workgroup barrier)
    (1, False, 64, 64, 35, "f32"),
    (1, True, 100, 128, 9, "f32"),
    (2, False, 33, 100, 12, "f32"),
    (1, False, 20, 17, 5, "f32"),       # two workgroups, the second nearly empty
    (1, False, 128, 96, 1, "f32"),      # T = 1: nothing is exchanged
    (2, True, 70, 80, 7, "bf16"),
])
def test_small_dense_widths_every_wave_on_its_own(shape, monkeypatch):
    L, bidir, D, H, T, dtype = shape
    case = inputs.make_case(_wl(96, L, bidir, D, H, T, 1, dtype=dtype, a=0.3 if dtype == "f32" else 0.1), k=H + T, random_state=True)
    for coop in (True, False):
        desc, _ = check_case(case, DENSE, PERSIST, cooperative=coop)
        assert "persist_b1-dense" in desc
    on, _ = run_gpu(case, DENSE, PERSIST)
    monkeypatch.setenv("LSTM355_L2_HANDOVER", "0")
    off, _ = run_gpu(case, DENSE, PERSIST)
    monkeypatch.delenv("LSTM355_L2_HANDOVER")
    for a, b in zip(on, off):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_projection_density_switch(monkeypatch):
    """LSTM355_SPARSE_PROJ_MAX_DENSITY at lstm_create moves the boundary between the projection over the kept entries and
    the dense matrix-core product; both meet the oracle (they differ from each other only in summation order)."""
    case = inputs.make_case(_wl(94, 1, True, 320, 256, 8, 40, keep=0.12), k=2, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    assert "proj=q16" in desc
    monkeypatch.setenv("LSTM355_SPARSE_PROJ_MAX_DENSITY", "0")
    desc, _ = check_case(case, CSR, PAUTO)
    monkeypatch.delenv("LSTM355_SPARSE_PROJ_MAX_DENSITY")
    assert "proj=dense" in desc
    case = inputs.make_case(_wl(94, 1, False, 320, 256, 8, 40, keep=0.3), k=3, random_state=True)
    desc, _ = check_case(case, CSR, PAUTO)
    assert "proj=dense" in desc      # above the default fraction
    monkeypatch.setenv("LSTM355_SPARSE_PROJ_MAX_DENSITY", "0.5")
    desc, _ = check_case(case, CSR, PAUTO)
    monkeypatch.delenv("LSTM355_SPARSE_PROJ_MAX_DENSITY")
    assert "proj=q16" in desc


def test_wide_dense_bidirectional_batch1():
    """Both directions of a dense batch-1 layer too wide for the fused input side: a projection launch per direction
    (the stream over the fragment-ordered weights) and the persistent recurrence."""
    case = inputs.make_case(_wl(96, 1, True, 200, 1344, 6, 1, a=0.05), k=5, random_state=True)
    desc, _ = check_case(case, DENSE, PAUTO)
    assert desc.count("proj=dense,rec=persist_b1-dense") == 2, desc


def test_few_input_rows_take_the_dense_projection_down_to_a_few_percent_kept():
    """With at most 64 input rows a separate projection launch of a row-compressed W_x streams the fragment-ordered
    dense copy on the matrix cores unless fewer than 4 % of the weights are kept; both choices meet the oracle."""
    for keep, want in ((0.3, "proj=dense"), (0.02, "proj=csr")):
        for T, Bn in ((9, 1), (5, 7), (15, 4)):
            case = inputs.make_case(_wl(95, 2, True, 72, 100, T, Bn, keep=keep), k=T + Bn, random_state=True)
            desc, _ = check_case(case, CSR, STEP)
            assert want in desc, desc


@pytest.mark.parametrize("which", ["mask_h_empty", "mask_x_empty", "both_empty", "rows_and_columns_gone", "all_kept_compressed"])
@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, T, B
    (2, False, 40, 130, 6, 1),      # batch 1: two-layer wavefront / register-resident slices
    (1, True, 33, 72, 5, 3),        # small batch: quarter-wave recurrence, projection over few rows
    (2, True, 64, 96, 12, 8),       # enough input rows for the projection over the kept entries
])
def test_degenerate_masks(which, shape):
    """What grow-and-prune can leave behind: a matrix with nothing kept, rows and columns pruned away entirely (Section 4,
    row/column pruning), and a mask that keeps everything stored in the compressed form.  Every format and plan against
    the oracle on the same masks."""
    L, bidir, D, H, T, Bn = shape
    case = inputs.make_case(_wl(97, L, bidir, D, H, T, Bn, keep=0.3), k=len(which) + H, random_state=True)
    for p in case.weights.values():
        if which in ("mask_h_empty", "both_empty"):
            p["Mh"][:] = 0
        if which in ("mask_x_empty", "both_empty"):
            p["Mx"][:] = 0
        if which == "rows_and_columns_gone":
            for M in (p["Mx"], p["Mh"]):
                M[::3, :] = 0               # every third row of the stacked matrix (all gates of some units, single gates of others)
                M[:, 1::4] = 0
            p["Mh"][0:H, :] = 0            # the whole forget gate of the recurrent matrix
        if which == "all_kept_compressed":
            p["Mx"][:] = 1
            p["Mh"][:] = 1
    for fmt in (DENSE, CSR):
        for plan in (PAUTO, STEP):
            check_case(case, fmt, plan)


@pytest.mark.parametrize("Bn", [1, 4])
@pytest.mark.parametrize("fmt", [DENSE, CSR])
def test_wider_than_any_persistent_kernel(Bn, fmt):
    """A layer wider than the on-chip-resident kernels take (their LDS copy of h ends at 64 KB, the dense batch-1 kernel
    at 2048 units): the planner falls back to one launch per step and the result still meets the oracle."""
    case = inputs.make_case(_wl(98, 1, False, 48, 6200 if fmt == CSR else 2304, 3, Bn, a=0.02, keep=0.02 if fmt == CSR else None), k=Bn, random_state=True)
    desc, _ = check_case(case, fmt, PAUTO)
    assert "stepwise" in desc, desc


@pytest.mark.parametrize("shape", [
    # L, bidir, D, H, T, B -- dense fp32 layers at small and medium batch: W_h as matrix-instruction fragments in registers
    (1, False, 40, 72, 6, 3),        # one 16-row block, nine workgroups, the last with one unit
    (2, True, 33, 100, 5, 16),
    (1, True, 64, 200, 7, 20),       # two row blocks, the second ragged
    (1, False, 48, 330, 4, 40),      # three row blocks
    (1, False, 32, 520, 3, 64),      # four row blocks of 16 would exceed the grid: two of 32
    (1, False, 24, 1100, 3, 5),      # twelve k-blocks per wave
    (1, False, 16, 1530, 2, 2),      # the widest layer the kernel takes (k-blocks of a wave in registers)
    (3, True, 20, 50, 9, 130),       # nine row blocks
    (1, False, 8, 3, 4, 2),          # three units: one workgroup, most of its waves without a k-block
    (1, True, 24, 500, 3, 96),       # the grid only fits with three 16-row blocks per workgroup
    (1, True, 24, 500, 2, 128),      # ... with four
    (2, True, 40, 256, 6, 100),      # eight groups of 32 workgroups, each group on one XCD
    (1, False, 24, 1500, 2, 20),     # twelve k-blocks per wave take one 16-row block only: two runs of ten batch columns
    (1, True, 24, 1500, 2, 9),       # both directions need more workgroups than there are compute units: a launch each
    (2, True, 24, 800, 2, 100),      # ... and runs of batch columns on top, in both layers
])
def test_dense_small_batch_persistent(shape):
    L, bidir, D, H, T, Bn = shape
    for rs in (False, True):
        case = inputs.make_case(_wl(99, L, bidir, D, H, T, Bn, a=min(0.3, 1.5 / np.sqrt(max(H, D)))), k=H + Bn, random_state=rs)
        for coop in (True, False):
            desc, _ = check_case(case, DENSE, PAUTO, cooperative=coop)
            assert "rec=persist-dense-f32" in desc, desc
    check_case(case, DENSE, STEP)


def test_yardsticks_run_and_are_plausible():
    """The achievable-peak yardsticks: matrix-instruction issue loops, the streaming copy and the data-free barrier."""
    import torch
    bf16, ghz = B.lstm_bench_mfma(B.LSTM_BF16, reps=2000, iters=2, with_clock=True)
    f32 = B.lstm_bench_mfma(B.LSTM_F32, reps=2000, iters=2)
    assert 500 < bf16 < 2600 and 30 < f32 < 165, (bf16, f32)     # below the spec-sheet peaks, above a third of them
    assert 0.5 < ghz < 2.6, ghz
    rnd, ghz_r = B.lstm_bench_mfma(B.LSTM_BF16, reps=2000, iters=2, random_operands=True, with_clock=True)
    assert 500 < rnd <= bf16 * 1.05 and 0.5 < ghz_r < 2.6, (rnd, ghz_r)
    assert 30 < B.lstm_bench_mfma(B.LSTM_F32, reps=2000, iters=2, random_operands=True) < 165
    n = 1 << 28
    src = torch.arange(n // 4, dtype=torch.int32, device="cuda:0")
    dst = torch.zeros_like(src)
    us = B.lstm_bench_copy(dst.data_ptr(), src.data_ptr(), n, 3)
    assert torch.equal(src, dst)
    assert 1000 < 2 * n / us / 1e3 < 8000, us                    # GB/s, read + write
    m = 4096 + 16 * 37                                           # a size with a ragged tail for the unrolled loop
    d2 = torch.zeros(m // 4, dtype=torch.int32, device="cuda:0")
    B.lstm_bench_copy(d2.data_ptr(), src.data_ptr(), m, 1)
    assert torch.equal(d2, src[: m // 4])
    for coop in (False, True):
        us = B.lstm_bench_barrier(256, 12, steps=100, iters=2, cooperative=coop)
        assert 0.1 < us < 20, us
    with pytest.raises(B.LstmError):
        B.lstm_bench_barrier(257, 12)
    with pytest.raises(B.LstmError):
        B.lstm_bench_mfma(7)
