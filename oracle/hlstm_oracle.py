"""ctypes front-end of the C oracle in hlstm_oracle.c.  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file (cell equations of the paper's Section 4 with one
ReLU hidden layer per gate, masks per the mask-based approach of Section 4, stacking and
directions per Section 5).  This wrapper only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
from typing import Dict, Optional, Tuple

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        PP = ctypes.POINTER(ctypes.c_void_p)
        lib.hlstm_oracle_forward.restype = ctypes.c_int
        lib.hlstm_oracle_forward.argtypes = [ctypes.c_int] * 7 + [PP] * 8 + [ctypes.c_void_p] * 6 + [ctypes.c_int]
        _lib = lib
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def forward(weights: Dict[Tuple[int, int], Dict[str, Optional[np.ndarray]]],
            x: np.ndarray, h0: Optional[np.ndarray] = None, c0: Optional[np.ndarray] = None,
            *, layers: int, ndir: int, hidden: int, gate_hidden: int, nthreads: int = 0):
    """Run the oracle.  weights[(l, d)] = dict(W1x, M1x|None, W1h, M1h|None, b1, W2, M2|None, b2);
    gate rows f,i,o,g (W1x/W1h/b1: row q*G + g; W2/b2: row q*H + j).

    x [T,B,D0] (fp32 values), h0/c0 [L*ndir,B,H] or None.  Returns (y, hT, cT) in float64.
    """
    lib = _load()
    x = _f32(x)
    T, B, D0 = x.shape
    H, G = hidden, gate_hidden
    n = layers * ndir
    keep = []

    def ptr_array(key, dtype, shape_of, required):
        arr = (ctypes.c_void_p * n)()
        for l in range(layers):
            D = D0 if l == 0 else ndir * H
            for d in range(ndir):
                a = weights[(l, d)].get(key)
                if a is None:
                    if required:
                        raise ValueError(f"{key} of layer {l} direction {d} missing")
                    arr[l * ndir + d] = None
                    continue
                a = np.ascontiguousarray(a, dtype=dtype)
                want = shape_of(D)
                if a.shape != want:
                    raise ValueError(f"{key}[{l},{d}] has shape {a.shape}, expected {want}")
                keep.append(a)
                arr[l * ndir + d] = a.ctypes.data
        return arr

    W1x = ptr_array("W1x", np.float32, lambda D: (4 * G, D), True)
    M1x = ptr_array("M1x", np.uint8, lambda D: (4 * G, D), False)
    W1h = ptr_array("W1h", np.float32, lambda D: (4 * G, H), True)
    M1h = ptr_array("M1h", np.uint8, lambda D: (4 * G, H), False)
    b1 = ptr_array("b1", np.float32, lambda D: (4 * G,), True)
    W2 = ptr_array("W2", np.float32, lambda D: (4 * H, G), True)
    M2 = ptr_array("M2", np.uint8, lambda D: (4 * H, G), False)
    b2 = ptr_array("b2", np.float32, lambda D: (4 * H,), True)
    if h0 is not None:
        h0 = _f32(h0)
        assert h0.shape == (n, B, H)
    if c0 is not None:
        c0 = _f32(c0)
        assert c0.shape == (n, B, H)
    y = np.zeros((T, B, ndir * H), dtype=np.float64)
    hT = np.zeros((n, B, H), dtype=np.float64)
    cT = np.zeros((n, B, H), dtype=np.float64)
    PP = ctypes.POINTER(ctypes.c_void_p)
    rc = lib.hlstm_oracle_forward(
        layers, ndir, D0, H, G, T, B,
        ctypes.cast(W1x, PP), ctypes.cast(M1x, PP), ctypes.cast(W1h, PP), ctypes.cast(M1h, PP), ctypes.cast(b1, PP),
        ctypes.cast(W2, PP), ctypes.cast(M2, PP), ctypes.cast(b2, PP),
        x.ctypes.data, None if h0 is None else h0.ctypes.data, None if c0 is None else c0.ctypes.data,
        y.ctypes.data, hT.ctypes.data, cT.ctypes.data, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"hlstm_oracle_forward failed ({rc})")
    return y, hT, cT


def forward_case(case, nthreads: int = 0):
    """Oracle on a seeded H-LSTM case object (duck-typed: .w.layers/.w.ndir/.w.hidden/.w.gate_hidden, ...)."""
    w = case.w
    return forward(case.weights, case.x, case.h0, case.c0, layers=w.layers, ndir=w.ndir, hidden=w.hidden,
                   gate_hidden=w.gate_hidden, nthreads=nthreads)
