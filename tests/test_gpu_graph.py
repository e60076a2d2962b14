"""A forward recorded into a HIP graph: every replay, with eager forwards and synchronisations between the replays, gives
the bits of the eager forward (the exchange tags restart inside the graph; nothing of a replay leaks into eager calls
and the other way round)."""
import numpy as np
import pytest

from paper_1901_10997_amd import binding as B
from paper_1901_10997_amd import inputs
from parity_util import check_case, run_gpu

pytestmark = pytest.mark.gpu


def _wl(cid, L, bidir, D, H, T, Bn, dtype="f32", a=0.3, keep=None, gate_hidden=0):
    return inputs.Workload(cid, f"graph_L{L}_D{D}_H{H}_T{T}_B{Bn}", L, bidir, D, H, T, Bn, dtype, a, keep, "uniform", gate_hidden)


CASES = [
    # L, bidir, D, H, T, B, dtype, keep, G, expected in plan
    (2, False, 40, 96, 12, 1, "f32", 0.2, 0, "wavefront"),          # batch 1, two layers per launch, handle-owned slots
    (2, True, 24, 80, 9, 1, "f32", None, 0, "persist_b1-dense"),    # batch 1, dense, both directions
    (1, True, 24, 96, 15, 4, "f32", 0.2, 0, "persist_batched"),     # small batch, workspace-owned slots
    (1, True, 64, 128, 6, 64, "f32", None, 0, "persist-dense-f32"), # dense fp32 at medium batch, flags cleared inside the graph
    (1, False, 48, 800, 4, 64, "f32", 0.1, 0, "batch/"),            # a layer cut into runs of batch columns, a launch each
    (1, False, 24, 2304, 3, 2, "f32", None, 0, "stepwise"),         # wider than any resident kernel: one launch per step
    (1, False, 32, 64, 10, 1, "f32", 0.2, 48, "persist_b1-hlstm"),  # H-LSTM, batch 1
    (1, True, 32, 64, 8, 4, "f32", 0.2, 48, "persist_batched-hlstm"),               # H-LSTM, small batch
    (1, False, 256, 256, 6, 64, "bf16", None, 0, ""),               # bf16, large batch
]


@pytest.mark.parametrize("L,bidir,D,H,T,Bn,dtype,keep,G,expect", CASES)
def test_graph_replays_match_eager(L, bidir, D, H, T, Bn, dtype, keep, G, expect):
    import torch
    case = inputs.make_case(_wl(95, L, bidir, D, H, T, Bn, dtype, keep=keep, gate_hidden=G), 2, random_state=True)
    check_case(case)                                                     # eager forward against the oracle
    eager, desc, model = run_gpu(case, return_model=True)                # the same bits again, and the warm-up
    assert expect in desc, desc
    dev = torch.device("cuda:0")
    xdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    xa = torch.from_numpy(case.x).to(dev).to(xdt)
    case_b = inputs.make_case(case.w, 3, random_state=True)
    case_b.weights = case.weights
    xb = torch.from_numpy(case_b.x).to(dev).to(xdt)
    h0, c0 = torch.from_numpy(case.h0).to(dev), torch.from_numpy(case.c0).to(dev)
    eager_b = [t.cpu().numpy() for t in model.forward(xb, h0, c0)]       # second input, same weights and state
    assert not np.array_equal(eager_b[0], eager[0])
    xs = xa.clone()                                                      # the graph's input buffer
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        outs = model.forward(xs, h0, c0, check=False)
    assert B.lstm_describe_plan(model.handle) == desc

    def same(want, got):
        for a, b in zip(want, got):
            assert np.array_equal(a, b.cpu().numpy())

    # replays alternate between the two inputs, so that whatever one replay leaves in the exchange slots would be wrong
    # for the next; eager forwards of the same handle run between them
    for rep in range(4):
        xs.copy_(xb if rep % 2 else xa)
        for o in outs:
            o.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        B.lstm_check(model.handle)
        same(eager_b if rep % 2 else eager, outs)
        same(eager_b, model.forward(xb, h0, c0))
        same(eager, model.forward(xa, h0, c0))
    g.replay()                                                           # two replays back to back
    g.replay()
    torch.cuda.synchronize()
    B.lstm_check(model.handle)
    same(eager_b, outs)
    model.close()
