"""Seeded synthetic workloads for the stacked-LSTM forward pass.

This module only draws random numbers and shapes them; it contains none of the
LSTM arithmetic.  Both the CPU oracle's tests and the GPU parity tests take their
inputs from here so that the two sides see bit-identical host arrays.

Shapes follow the models of the paper's experiments (Section 5): a 2-layer
1500-wide language-model stack and a 5-layer bidirectional 800-wide speech stack,
with weight sparsity in the range the paper reports after weight pruning.  Values
are synthetic (uniform weights, Bernoulli masks, normal inputs).

Gate-row order of every weight matrix is f, i, o, g (the order in which the paper
stacks the four gates in its cell equations, Section 4): rows [0,H) forget,
[H,2H) input, [2H,3H) output, [3H,4H) cell candidate.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

SEED_BASE = 190110997


@dataclass(frozen=True)
class Workload:
    """Shape and value recipe of one synthetic LSTM workload."""
    cid: int                 # config number, enters the seed
    name: str
    layers: int
    bidirectional: bool
    input_dim: int
    hidden: int
    T: int
    B: int
    dtype: str = "f32"       # "f32" | "bf16" (bf16 = operands rounded to bf16 on the host)
    a: float = 0.1           # weights ~ U(-a, a)
    keep: Optional[float] = None   # Bernoulli keep-probability of the masks; None = dense (no masks)
    bias: str = "forget1"    # "forget1": 0 except forget gate 1.0 ; "uniform": U(-a, a)
    gate_hidden: int = 0     # > 0: H-LSTM cell, width of the hidden layer inside each gate

    @property
    def ndir(self) -> int:
        return 2 if self.bidirectional else 1

    def layer_input_dim(self, l: int) -> int:
        return self.input_dim if l == 0 else self.ndir * self.hidden


def c1() -> Workload:
    return Workload(1, "c1_small_dense", 1, False, 200, 200, 35, 1, "f32", 0.1, None, "forget1")


def c2(B: int = 1) -> Workload:
    return Workload(2, f"c2_lm_2x1500_b{B}", 2, False, 1500, 1500, 35, B, "f32", 0.04, 0.10, "uniform")


def c3(H: int) -> Workload:
    return Workload(3, f"c3_sweep_h{H}", 1, False, H, H, 35, 1, "f32", 0.1, None, "forget1")


def c3_hidden_sizes() -> List[int]:
    return list(range(64, 2048 + 1, 32))


def c4() -> Workload:
    return Workload(4, "c4_speech_5x800_bidir", 5, True, 640, 800, 300, 16, "f32", 0.035, 0.15, "uniform")


def c5() -> Workload:
    return Workload(5, "c5_throughput_2x1024_bf16", 2, False, 1024, 1024, 128, 256, "bf16", 0.03, None, "uniform")


def h1() -> Workload:
    """Language-model H-LSTM of the paper's Section 5.1: one layer, hidden state 1500, one hidden layer of width
    1500 per gate, word embeddings of width 400; masks keep 10 % (the pruned models keep 4-17 %)."""
    return Workload(6, "h1_lm_hlstm_1x1500_b1", 1, False, 400, 1500, 35, 1, "f32", 0.04, 0.10, "uniform", 1500)


def h2() -> Workload:
    """Speech H-LSTM of the paper's Section 5.2: three bidirectional layers, hidden state and gate hidden layers 800
    wide, batch 16; masks keep 20 % (the pruned models keep 27-40 % of a smaller dense model)."""
    return Workload(7, "h2_speech_hlstm_3x800_bidir", 3, True, 640, 800, 300, 16, "f32", 0.035, 0.20, "uniform", 800)


def shrink(w: Workload, **kw) -> Workload:
    """Same recipe at other sizes (used by tests that need the oracle to finish quickly)."""
    return replace(w, **kw)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays stored as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


@dataclass
class Case:
    """Host arrays of one seeded instance of a workload.

    weights[(l, d)] = dict(Wx[4H,D_l] f32, Mx u8 or None, Wh[4H,H] f32, Mh u8 or None, b[4H] f32)
    H-LSTM workloads (gate_hidden = G > 0) instead hold
    weights[(l, d)] = dict(W1x[4G,D_l], M1x, W1h[4G,H], M1h, b1[4G], W2[4H,G], M2, b2[4H])
    x[T,B,D0] f32 ; h0, c0 [L*ndir, B, H] f32 or None (= zeros)
    """
    w: Workload
    seed: int
    weights: Dict[Tuple[int, int], Dict[str, Optional[np.ndarray]]]
    x: np.ndarray
    h0: Optional[np.ndarray]
    c0: Optional[np.ndarray]


def make_case(w: Workload, k: int = 0, random_state: bool = False) -> Case:
    """Draw instance `k` of workload `w`.

    Draw order (fixed, so that a case is reproducible from (cid, k) alone):
    for each layer, for each direction: Wx, mask_x, Wh, mask_h, b (H-LSTM: W1x, mask_1x, W1h, mask_1h, b1, W2,
    mask_2, b2; forget-gate bias 1 applies to b2 when bias == "forget1"); then x; then, if `random_state`, h0 and
    c0 ~ U(-0.5, 0.5).
    """
    seed = SEED_BASE + 1000 * w.cid + k
    rng = np.random.Generator(np.random.PCG64(seed))
    H = w.hidden
    G = 4 * H
    weights: Dict[Tuple[int, int], Dict[str, Optional[np.ndarray]]] = {}
    for l in range(w.layers):
        D = w.layer_input_dim(l)
        for d in range(w.ndir):
            if w.gate_hidden > 0:
                R1 = 4 * w.gate_hidden

                def draw(shape):
                    Wm = rng.uniform(-w.a, w.a, shape).astype(np.float32)
                    Mm = (rng.random(shape) < w.keep).astype(np.uint8) if w.keep is not None else None
                    return Wm, Mm

                W1x, M1x = draw((R1, D))
                W1h, M1h = draw((R1, H))
                b1 = rng.uniform(-w.a, w.a, R1).astype(np.float32)
                W2, M2 = draw((G, w.gate_hidden))
                if w.bias == "forget1":
                    b2 = np.zeros(G, dtype=np.float32)
                    b2[0:H] = 1.0
                else:
                    b2 = rng.uniform(-w.a, w.a, G).astype(np.float32)
                weights[(l, d)] = dict(W1x=W1x, M1x=M1x, W1h=W1h, M1h=M1h, b1=b1, W2=W2, M2=M2, b2=b2)
                continue
            Wx = rng.uniform(-w.a, w.a, (G, D)).astype(np.float32)
            Mx = (rng.random((G, D)) < w.keep).astype(np.uint8) if w.keep is not None else None
            Wh = rng.uniform(-w.a, w.a, (G, H)).astype(np.float32)
            Mh = (rng.random((G, H)) < w.keep).astype(np.uint8) if w.keep is not None else None
            if w.bias == "forget1":
                b = np.zeros(G, dtype=np.float32)
                b[0:H] = 1.0
            elif w.bias == "uniform":
                b = rng.uniform(-w.a, w.a, G).astype(np.float32)
            else:
                raise ValueError(w.bias)
            if w.dtype == "bf16":
                Wx = round_to_bf16(Wx)
                Wh = round_to_bf16(Wh)
            weights[(l, d)] = dict(Wx=Wx, Mx=Mx, Wh=Wh, Mh=Mh, b=b)
    x = rng.standard_normal((w.T, w.B, w.input_dim)).astype(np.float32)
    if w.dtype == "bf16":
        x = round_to_bf16(x)
    h0 = c0 = None
    if random_state:
        n = w.layers * w.ndir
        h0 = rng.uniform(-0.5, 0.5, (n, w.B, H)).astype(np.float32)
        c0 = rng.uniform(-0.5, 0.5, (n, w.B, H)).astype(np.float32)
    return Case(w, seed, weights, x, h0, c0)


def select_batch(case: Case, cols: List[int]) -> Case:
    """The same case restricted to the given batch columns (sequences are independent)."""
    cols = list(cols)
    w = replace(case.w, B=len(cols))
    x = np.ascontiguousarray(case.x[:, cols, :])
    h0 = None if case.h0 is None else np.ascontiguousarray(case.h0[:, cols, :])
    c0 = None if case.c0 is None else np.ascontiguousarray(case.c0[:, cols, :])
    return Case(w, case.seed, case.weights, x, h0, c0)


def structure_masks(case: Case, unit_frac: float, input_frac: float, k: int = 0, gate_unit_frac: Optional[float] = None):
    """The same case after a row/column pruning outcome has been stamped onto its masks.

    In every (layer, direction) a random subset of round(unit_frac * H) hidden units survives (of one size per layer,
    the sets differ; unit_frac may be a list with one fraction per layer), and round(input_frac * D0) of the input
    features; in an H-LSTM workload also
    round(gate_unit_frac * G) of the hidden-layer units inside the gates (the same index set for the four gates of a
    cell; default: unit_frac).  A connection stays active iff the case's own mask keeps it (dense workloads: every
    connection), its row belongs to a surviving unit and its column to a surviving source (input feature, unit of
    the layer below, the layer's own unit for a recurrent matrix, hidden-layer unit of the same gate for a gate-output
    matrix) - the pattern of the paper's figure on the mask of an input-to-hidden matrix after the row/column phase.
    Returns (case with the new masks, units[(l, d)] sorted int arrays, inputs sorted int array); H-LSTM workloads:
    (case, units, inputs, gate_units[(l, d)]).
    """
    w = case.w
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 7777 * w.cid + 31 * k + 5))
    H, D0, G = w.hidden, w.input_dim, w.gate_hidden
    fracs = [unit_frac] * w.layers if np.isscalar(unit_frac) else list(unit_frac)   # one per layer when a list
    assert len(fracs) == w.layers
    Dc = max(1, int(round(input_frac * D0)))
    feats = np.sort(rng.permutation(D0)[:Dc]).astype(np.int64)
    units = {}
    for l in range(w.layers):
        Hc = max(1, int(round(fracs[l] * H)))
        for d in range(w.ndir):
            units[(l, d)] = np.sort(rng.permutation(H)[:Hc]).astype(np.int64)
    gate_units = {}
    if G > 0:
        for l in range(w.layers):
            Gc = max(1, int(round((fracs[l] if gate_unit_frac is None else gate_unit_frac) * G)))
            for d in range(w.ndir):
                gate_units[(l, d)] = np.sort(rng.permutation(G)[:Gc]).astype(np.int64)

    def stamp(M, shape, rows, cols):
        out = np.ones(shape, np.uint8) if M is None else M.copy()
        out[~rows, :] = 0
        out[:, ~cols] = 0
        return out

    weights = {}
    for l in range(w.layers):
        D = w.layer_input_dim(l)
        src = np.zeros(D, dtype=bool)
        if l == 0:
            src[feats] = True
        else:
            for d in range(w.ndir):
                src[d * H + units[(l - 1, d)]] = True
        for d in range(w.ndir):
            cur = case.weights[(l, d)]
            rows = np.zeros(H, dtype=bool)
            rows[units[(l, d)]] = True
            rows4 = np.tile(rows, 4)
            if G > 0:
                grow = np.zeros(G, dtype=bool)
                grow[gate_units[(l, d)]] = True
                grow4 = np.tile(grow, 4)
                weights[(l, d)] = dict(W1x=cur["W1x"], M1x=stamp(cur["M1x"], (4 * G, D), grow4, src),
                                       W1h=cur["W1h"], M1h=stamp(cur["M1h"], (4 * G, H), grow4, rows), b1=cur["b1"],
                                       W2=cur["W2"], M2=stamp(cur["M2"], (4 * H, G), rows4, grow), b2=cur["b2"])
            else:
                weights[(l, d)] = dict(Wx=cur["Wx"], Mx=stamp(cur["Mx"], (4 * H, D), rows4, src),
                                       Wh=cur["Wh"], Mh=stamp(cur["Mh"], (4 * H, H), rows4, rows), b=cur["b"])
    out = Case(w, case.seed, weights, case.x, case.h0, case.c0)
    if G > 0:
        return out, units, feats, gate_units
    return out, units, feats


def matmul_operands(n: int, batch: int, keep: Optional[float], seed: int = 0):
    """Operands of the stand-alone product of the paper's Section 3 (dense input batch times a square weight matrix
    of dimension n, of which a fraction `keep` is kept): X [batch, n] ~ N(0,1), W [n, n] ~ U(-0.1, 0.1), mask
    Bernoulli(keep) as uint8, or None for a dense matrix.  Draw order: W, mask, X."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 1000 * 8 + seed))
    W = rng.uniform(-0.1, 0.1, (n, n)).astype(np.float32)
    M = None if keep is None else (rng.random((n, n)) < keep).astype(np.uint8)
    X = rng.standard_normal((batch, n)).astype(np.float32)
    return X, W, M


def make_layers_case(input_dim: int, hiddens: List[int], bidirectional: bool, T: int, B: int, a: float = 0.3,
                     keep: Optional[float] = None, gate_hiddens: Optional[List[int]] = None, k: int = 0,
                     random_state: bool = True):
    """A stack whose layers have their own widths (what row/column pruning of the paper's Section 4 leaves behind:
    every layer shrinks by its own amount).  Draw order as make_case, with layer l's shapes.
    Returns (weights[(l, d)], x[T,B,input_dim], h0 list, c0 list): h0[n], c0[n] are [B, hiddens[l]] for n = l*ndir + d,
    or None when random_state is off."""
    ndir = 2 if bidirectional else 1
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 1000 * 9 + k))
    weights: Dict[Tuple[int, int], Dict[str, Optional[np.ndarray]]] = {}

    def draw(shape):
        Wm = rng.uniform(-a, a, shape).astype(np.float32)
        Mm = (rng.random(shape) < keep).astype(np.uint8) if keep is not None else None
        return Wm, Mm

    for l, H in enumerate(hiddens):
        D = input_dim if l == 0 else ndir * hiddens[l - 1]
        for d in range(ndir):
            if gate_hiddens is not None:
                G = gate_hiddens[l]
                W1x, M1x = draw((4 * G, D))
                W1h, M1h = draw((4 * G, H))
                b1 = rng.uniform(-a, a, 4 * G).astype(np.float32)
                W2, M2 = draw((4 * H, G))
                b2 = rng.uniform(-a, a, 4 * H).astype(np.float32)
                weights[(l, d)] = dict(W1x=W1x, M1x=M1x, W1h=W1h, M1h=M1h, b1=b1, W2=W2, M2=M2, b2=b2)
            else:
                Wx, Mx = draw((4 * H, D))
                Wh, Mh = draw((4 * H, H))
                b = rng.uniform(-a, a, 4 * H).astype(np.float32)
                weights[(l, d)] = dict(Wx=Wx, Mx=Mx, Wh=Wh, Mh=Mh, b=b)
    x = rng.standard_normal((T, B, input_dim)).astype(np.float32)
    h0 = c0 = None
    if random_state:
        h0 = [rng.uniform(-0.5, 0.5, (B, hiddens[n // ndir])).astype(np.float32) for n in range(len(hiddens) * ndir)]
        c0 = [rng.uniform(-0.5, 0.5, (B, hiddens[n // ndir])).astype(np.float32) for n in range(len(hiddens) * ndir)]
    return weights, x, h0, c0
