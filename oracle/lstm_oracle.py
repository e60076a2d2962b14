"""ctypes front-end of the C oracle in lstm_oracle.c.  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file (cell equations of the paper's Section 4 with zero
hidden layers per gate, masks per the mask-based approach of Section 4, stacking and
directions per Section 5).  This wrapper only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        PP = ctypes.POINTER(ctypes.c_void_p)
        lib.lstm_oracle_forward.restype = ctypes.c_int
        lib.lstm_oracle_forward.argtypes = [ctypes.c_int] * 6 + [PP] * 5 + [ctypes.c_void_p] * 6 + [ctypes.c_int]
        lib.lstm_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().lstm_oracle_max_threads())


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def forward(weights: Dict[Tuple[int, int], Dict[str, Optional[np.ndarray]]],
            x: np.ndarray, h0: Optional[np.ndarray] = None, c0: Optional[np.ndarray] = None,
            *, layers: int, ndir: int, hidden: int, nthreads: int = 0):
    """Run the oracle.  weights[(l, d)] = dict(Wx, Mx|None, Wh, Mh|None, b); gate rows f,i,o,g.

    x [T,B,D0] (fp32 values), h0/c0 [L*ndir,B,H] or None.  Returns (y, hT, cT) in float64.
    """
    lib = _load()
    x = _f32(x)
    T, B, D0 = x.shape
    H = hidden
    n = layers * ndir
    keep = []  # keep converted arrays alive during the call

    def ptr_array(key, dtype, shape_of):
        arr = (ctypes.c_void_p * n)()
        any_set = False
        for l in range(layers):
            D = D0 if l == 0 else ndir * H
            for d in range(ndir):
                a = weights[(l, d)].get(key)
                if a is None:
                    arr[l * ndir + d] = None
                    continue
                a = np.ascontiguousarray(a, dtype=dtype)
                want = shape_of(D)
                if a.shape != want:
                    raise ValueError(f"{key}[{l},{d}] has shape {a.shape}, expected {want}")
                keep.append(a)
                arr[l * ndir + d] = a.ctypes.data
                any_set = True
        return arr, any_set

    Wx, _ = ptr_array("Wx", np.float32, lambda D: (4 * H, D))
    Mx, _ = ptr_array("Mx", np.uint8, lambda D: (4 * H, D))
    Wh, _ = ptr_array("Wh", np.float32, lambda D: (4 * H, H))
    Mh, _ = ptr_array("Mh", np.uint8, lambda D: (4 * H, H))
    bb, _ = ptr_array("b", np.float32, lambda D: (4 * H,))
    for l in range(layers):
        for d in range(ndir):
            if Wx[l * ndir + d] is None or Wh[l * ndir + d] is None or bb[l * ndir + d] is None:
                raise ValueError(f"weights of layer {l} direction {d} incomplete")
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
    rc = lib.lstm_oracle_forward(
        layers, ndir, D0, H, T, B,
        ctypes.cast(Wx, PP), ctypes.cast(Mx, PP), ctypes.cast(Wh, PP), ctypes.cast(Mh, PP), ctypes.cast(bb, PP),
        x.ctypes.data, None if h0 is None else h0.ctypes.data, None if c0 is None else c0.ctypes.data,
        y.ctypes.data, hT.ctypes.data, cT.ctypes.data, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"lstm_oracle_forward failed ({rc})")
    return y, hT, cT


def forward_case(case, nthreads: int = 0):
    """Oracle on a seeded case object (duck-typed: .w.layers/.w.ndir/.w.hidden, .weights, .x, .h0, .c0)."""
    w = case.w
    return forward(case.weights, case.x, case.h0, case.c0,
                   layers=w.layers, ndir=w.ndir, hidden=w.hidden, nthreads=nthreads)
