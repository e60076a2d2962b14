"""Shared helpers of the GPU parity tests: run a seeded case through the C ABI and compare with the oracle.

Tolerances (written here once):
  fp32 models : per output tensor, max |d| <= 1e-5  and  ||d||_2 / ||ref||_2 <= 1e-4
  bf16 models : per output tensor, ||d||_inf / ||ref||_inf <= 2e-2  and  ||d||_2 / ||ref||_2 <= 2e-2
where d = gpu - oracle and the oracle (fp64) sees the same host arrays (bf16 models: already bf16-rounded).
"""
from __future__ import annotations

import numpy as np

from oracle import hlstm_oracle as horc
from oracle import lstm_oracle as orc
from paper_1901_10997_amd import binding as B
from paper_1901_10997_amd import inputs

F32_MAX_ABS = 1e-5
F32_REL_L2 = 1e-4
BF16_REL = 2e-2


def run_gpu(case, fmt=B.LSTM_FMT_AUTO, plan=B.LSTM_PLAN_AUTO, waves=0, model=None, return_model=False, cooperative=True):
    import torch
    w = case.w
    dtype = B.LSTM_BF16 if w.dtype == "bf16" else B.LSTM_F32
    own = model is None
    if own:
        model = B.Lstm(w.layers, w.input_dim, w.hidden, w.bidirectional, dtype, gate_hidden=w.gate_hidden)
        model.set_weights_from(case.weights, fmt)
    B.lstm_set_plan(model.handle, plan, waves)
    B.lstm_set_launch_mode(model.handle, cooperative)
    dev = torch.device("cuda:0")
    x = torch.from_numpy(case.x).to(dev)
    if dtype == B.LSTM_BF16:
        x = x.to(torch.bfloat16)
    h0 = None if case.h0 is None else torch.from_numpy(case.h0).to(dev)
    c0 = None if case.c0 is None else torch.from_numpy(case.c0).to(dev)
    y, hT, cT = model.forward(x.contiguous(), h0, c0)
    out = (y.cpu().numpy(), hT.cpu().numpy(), cT.cpu().numpy())
    desc = B.lstm_describe_plan(model.handle)
    if return_model:
        return out, desc, model
    if own:
        model.close()
    return out, desc


def compare(gpu, ref, dtype: str, label: str = ""):
    """Assert the tolerance of the module docstring for each of (y, hT, cT); returns the worst figures."""
    worst = {}
    for name, g, r in zip(("y", "hT", "cT"), gpu, ref):
        g = np.asarray(g, dtype=np.float64)
        r = np.asarray(r, dtype=np.float64)
        assert g.shape == r.shape, (label, name, g.shape, r.shape)
        assert np.all(np.isfinite(g)), (label, name, "non-finite output")
        if g.size == 0:
            continue
        d = g - r
        max_abs = float(np.max(np.abs(d)))
        rel_l2 = float(np.linalg.norm(d) / max(np.linalg.norm(r), 1e-300))
        rel_inf = float(max_abs / max(np.max(np.abs(r)), 1e-300))
        worst[name] = (max_abs, rel_l2, rel_inf)
        if dtype == "bf16":
            assert rel_inf <= BF16_REL and rel_l2 <= BF16_REL, (label, name, max_abs, rel_l2, rel_inf)
        else:
            assert max_abs <= F32_MAX_ABS and rel_l2 <= F32_REL_L2, (label, name, max_abs, rel_l2)
    return worst


def check_case(case, fmt=B.LSTM_FMT_AUTO, plan=B.LSTM_PLAN_AUTO, waves=0, oracle_cols=None, label="", cooperative=True):
    """GPU on the whole case; oracle on the whole case or on the sampled batch columns `oracle_cols`."""
    print(f"[parity] {label or case.w.name} seed={case.seed} fmt={fmt} plan={plan} waves={waves} "
          f"L={case.w.layers} Dn={case.w.ndir} D={case.w.input_dim} H={case.w.hidden} G={case.w.gate_hidden} "
          f"T={case.w.T} B={case.w.B}",
          flush=True)
    gpu, desc = run_gpu(case, fmt, plan, waves, cooperative=cooperative)
    oracle_forward = horc.forward_case if case.w.gate_hidden > 0 else orc.forward_case
    if oracle_cols is None:
        ref = oracle_forward(case)
    else:
        sub = inputs.select_batch(case, oracle_cols)
        ref = oracle_forward(sub)
        gpu = (gpu[0][:, oracle_cols], gpu[1][:, oracle_cols], gpu[2][:, oracle_cols])
    worst = compare(gpu, ref, case.w.dtype, label or case.w.name)
    print(f"[parity]   plan={desc} worst={worst}", flush=True)
    return desc, worst
