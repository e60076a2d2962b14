"""ctypes binding of liblstm355 (include/lstm355.h).  Argument marshalling only: every step of the
forward pass runs in the library's HIP kernels.  There is no CPU fallback; if the shared library is
missing, loading raises.

Function names mirror the C ABI.  Device buffers are passed as integer addresses (e.g. the
``data_ptr()`` of a torch tensor); host arrays are numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

LSTM_F32, LSTM_BF16 = 0, 1
LSTM_OK = 0
LSTM_ERR_ARG, LSTM_ERR_SHAPE, LSTM_ERR_STATE, LSTM_ERR_NOMEM, LSTM_ERR_LAUNCH, LSTM_ERR_TIMEOUT = -1, -2, -3, -4, -5, -6
LSTM_FMT_AUTO, LSTM_FMT_DENSE_MASKED, LSTM_FMT_ROW_COMPRESSED = 0, 1, 2
LSTM_PLAN_AUTO, LSTM_PLAN_STEPWISE, LSTM_PLAN_PERSISTENT = 0, 1, 2

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblstm355.so")

# every symbol include/lstm355.h declares
EXPORTS = [
    "lstm_create", "lstm_create_h", "lstm_create_layers", "lstm_destroy", "lstm_last_error", "lstm_set_weights", "lstm_set_weights_h",
    "lstm_workspace_bytes",
    "lstm_forward", "lstm_check", "lstm_set_plan", "lstm_set_launch_mode", "lstm_set_default_launch_mode", "lstm_set_profiling", "lstm_get_profile", "lstm_describe_plan", "lstm_get_compressed",
    "lstm_latency_sweep", "lstm_latency_sweep_model", "lstm_find_lhp", "lstm_grow_to_lhp", "lstm_prune_weights", "lstm_prune_rows_cols", "lstm_prune_rows_cols_static",
    "lstm_compact_rows_cols",
    "lstm_bench_copy", "lstm_bench_matmul", "lstm_bench_mfma", "lstm_bench_barrier", "lstm_bench_exchange", "lstm_bench_group_exchange",
]

_lib = None


class LstmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"liblstm355 error {code}: {msg}")
        self.code = code


def load(build_if_missing: bool = True):
    """Load liblstm355.so; builds it with hipcc only when no built library is present."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, ci = c.c_void_p, c.c_int
    lib.lstm_create.restype = ci
    lib.lstm_create.argtypes = [ci, ci, ci, ci, ci, c.POINTER(vp)]
    lib.lstm_create_h.restype = ci
    lib.lstm_create_h.argtypes = [ci, ci, ci, ci, ci, ci, c.POINTER(vp)]
    lib.lstm_create_layers.restype = ci
    lib.lstm_create_layers.argtypes = [ci, ci, vp, vp, ci, ci, c.POINTER(vp)]
    lib.lstm_destroy.restype = ci
    lib.lstm_destroy.argtypes = [vp]
    lib.lstm_last_error.restype = c.c_char_p
    lib.lstm_last_error.argtypes = [vp]
    lib.lstm_set_weights.restype = ci
    lib.lstm_set_weights.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp, ci]
    lib.lstm_set_weights_h.restype = ci
    lib.lstm_set_weights_h.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, ci]
    lib.lstm_workspace_bytes.restype = c.c_size_t
    lib.lstm_workspace_bytes.argtypes = [vp, ci, ci]
    lib.lstm_forward.restype = ci
    lib.lstm_forward.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp, vp, vp, c.c_size_t, vp]
    lib.lstm_check.restype = ci
    lib.lstm_check.argtypes = [vp]
    lib.lstm_set_plan.restype = ci
    lib.lstm_set_plan.argtypes = [vp, ci, ci]
    lib.lstm_set_launch_mode.restype = ci
    lib.lstm_set_launch_mode.argtypes = [vp, ci]
    lib.lstm_set_default_launch_mode.restype = ci
    lib.lstm_set_default_launch_mode.argtypes = [ci]
    lib.lstm_set_profiling.restype = ci
    lib.lstm_set_profiling.argtypes = [vp, ci]
    lib.lstm_get_profile.restype = ci
    lib.lstm_get_profile.argtypes = [vp, c.POINTER(c.c_double), c.POINTER(ci), c.POINTER(c.c_double), c.POINTER(ci)]
    lib.lstm_describe_plan.restype = ci
    lib.lstm_describe_plan.argtypes = [vp, c.c_char_p, c.c_size_t]
    lib.lstm_get_compressed.restype = ci
    lib.lstm_get_compressed.argtypes = [vp, ci, ci, ci, c.POINTER(c.c_int64), vp, vp, vp]
    lib.lstm_latency_sweep.restype = ci
    lib.lstm_latency_sweep.argtypes = [vp, ci, ci, ci, ci, c.c_uint64, ci, ci, vp, vp, vp, vp, vp]
    lib.lstm_latency_sweep_model.restype = ci
    lib.lstm_latency_sweep_model.argtypes = [vp, vp, ci, ci, ci, ci, c.c_double, ci, ci, ci, c.c_uint64, ci, ci,
                                             vp, vp, vp, vp, vp]
    lib.lstm_grow_to_lhp.restype = ci
    lib.lstm_grow_to_lhp.argtypes = [vp, vp, ci, c.c_double, ci, c.POINTER(ci), c.POINTER(c.c_double)]
    lib.lstm_prune_weights.restype = ci
    lib.lstm_prune_weights.argtypes = [vp, vp, c.c_size_t, c.c_double, c.POINTER(c.c_size_t), c.POINTER(c.c_size_t), vp]
    lib.lstm_prune_rows_cols.restype = ci
    lib.lstm_prune_rows_cols.argtypes = [vp, vp, ci, ci, c.c_double, c.c_double, c.POINTER(ci), c.POINTER(ci), vp]
    lib.lstm_prune_rows_cols_static.restype = ci
    lib.lstm_prune_rows_cols_static.argtypes = [vp, vp, ci, ci, c.c_double, c.c_double, vp, vp]
    lib.lstm_compact_rows_cols.restype = ci
    lib.lstm_compact_rows_cols.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp, c.POINTER(ci), c.POINTER(ci), vp]
    lib.lstm_bench_mfma.restype = ci
    lib.lstm_bench_mfma.argtypes = [ci, ci, ci, ci, c.POINTER(c.c_double), c.POINTER(c.c_double), vp]
    lib.lstm_bench_barrier.restype = ci
    lib.lstm_bench_barrier.argtypes = [ci, ci, ci, ci, ci, c.POINTER(c.c_double), vp]
    lib.lstm_bench_matmul.restype = ci
    lib.lstm_bench_matmul.argtypes = [ci, ci, c.c_double, ci, c.c_uint64, ci, vp, vp, vp, c.POINTER(c.c_double), vp, vp]
    lib.lstm_find_lhp.restype = ci
    lib.lstm_find_lhp.argtypes = [vp, vp, ci, c.c_double, vp, c.POINTER(c.c_double)]
    lib.lstm_bench_copy.restype = ci
    lib.lstm_bench_copy.argtypes = [vp, vp, c.c_size_t, ci, c.POINTER(c.c_double), vp]
    lib.lstm_bench_exchange.restype = ci
    lib.lstm_bench_exchange.argtypes = [ci, ci, ci, ci, ci, c.POINTER(c.c_double), vp]
    lib.lstm_bench_group_exchange.restype = ci
    lib.lstm_bench_group_exchange.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, c.POINTER(c.c_double), c.POINTER(ci), vp]
    _lib = lib
    return lib


def _err(handle) -> str:
    s = load().lstm_last_error(handle)
    return s.decode() if s else ""


def _check(rc: int, handle=None):
    if rc != LSTM_OK:
        raise LstmError(rc, _err(handle))


def _host(a, dtype) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def lstm_create(layers: int, input_dim: int, hidden_dim: int, bidirectional: bool, dtype: int = LSTM_F32):
    h = ctypes.c_void_p()
    _check(load().lstm_create(layers, input_dim, hidden_dim, int(bool(bidirectional)), dtype, ctypes.byref(h)))
    return h


def lstm_create_h(layers: int, input_dim: int, hidden_dim: int, gate_hidden_dim: int, bidirectional: bool,
                  dtype: int = LSTM_F32):
    h = ctypes.c_void_p()
    _check(load().lstm_create_h(layers, input_dim, hidden_dim, gate_hidden_dim, int(bool(bidirectional)), dtype,
                                ctypes.byref(h)))
    return h


def lstm_create_layers(input_dim: int, hidden_dims: Sequence[int], gate_hidden_dims: Optional[Sequence[int]],
                       bidirectional: bool, dtype: int = LSTM_F32):
    """A stack whose layers have their own hidden widths (and, for H-LSTM cells, their own gate hidden widths)."""
    hs = np.ascontiguousarray(hidden_dims, dtype=np.int32)
    gs = None if gate_hidden_dims is None else np.ascontiguousarray(gate_hidden_dims, dtype=np.int32)
    if gs is not None and len(gs) != len(hs):
        raise ValueError("gate_hidden_dims and hidden_dims differ in length")
    h = ctypes.c_void_p()
    _check(load().lstm_create_layers(len(hs), input_dim, hs.ctypes.data, None if gs is None else gs.ctypes.data,
                                     int(bool(bidirectional)), dtype, ctypes.byref(h)))
    return h


def lstm_destroy(handle) -> None:
    _check(load().lstm_destroy(handle))


def lstm_set_weights(handle, layer: int, direction: int, Wx, mask_x, Wh, mask_h, b, fmt: int = LSTM_FMT_AUTO) -> None:
    Wx, Wh, b = _host(Wx, np.float32), _host(Wh, np.float32), _host(b, np.float32)
    mx, mh = _host(mask_x, np.uint8), _host(mask_h, np.uint8)
    if mx is not None and mx.shape != Wx.shape or mh is not None and mh.shape != Wh.shape:
        raise ValueError("mask shape differs from its weight matrix")
    _check(load().lstm_set_weights(handle, layer, direction, _p(Wx), _p(mx), _p(Wh), _p(mh), _p(b), fmt), handle)


def lstm_set_weights_h(handle, layer: int, direction: int, W1x, mask_1x, W1h, mask_1h, b1, W2, mask_2, b2,
                       fmt: int = LSTM_FMT_AUTO) -> None:
    W1x, W1h, b1 = _host(W1x, np.float32), _host(W1h, np.float32), _host(b1, np.float32)
    W2, b2 = _host(W2, np.float32), _host(b2, np.float32)
    m1x, m1h, m2 = _host(mask_1x, np.uint8), _host(mask_1h, np.uint8), _host(mask_2, np.uint8)
    for mk, wm in ((m1x, W1x), (m1h, W1h), (m2, W2)):
        if mk is not None and mk.shape != wm.shape:
            raise ValueError("mask shape differs from its weight matrix")
    _check(load().lstm_set_weights_h(handle, layer, direction, _p(W1x), _p(m1x), _p(W1h), _p(m1h), _p(b1),
                                     _p(W2), _p(m2), _p(b2), fmt), handle)


def lstm_workspace_bytes(handle, T: int, B: int) -> int:
    return int(load().lstm_workspace_bytes(handle, T, B))


def lstm_forward(handle, T: int, B: int, x_ptr: int, h0_ptr: Optional[int], c0_ptr: Optional[int], y_ptr: int,
                 hT_ptr: Optional[int], cT_ptr: Optional[int], ws_ptr: int, ws_bytes: int, stream: Optional[int] = None):
    _check(load().lstm_forward(handle, T, B, x_ptr, h0_ptr, c0_ptr, y_ptr, hT_ptr, cT_ptr, ws_ptr, ws_bytes, stream),
           handle)


def lstm_check(handle) -> None:
    _check(load().lstm_check(handle), handle)


def lstm_set_plan(handle, plan: int, waves_per_group: int = 0) -> None:
    _check(load().lstm_set_plan(handle, plan, waves_per_group), handle)


def lstm_set_launch_mode(handle, cooperative: bool) -> None:
    _check(load().lstm_set_launch_mode(handle, int(bool(cooperative))), handle)


def lstm_set_default_launch_mode(cooperative: bool) -> None:
    _check(load().lstm_set_default_launch_mode(int(bool(cooperative))))


def lstm_set_profiling(handle, enable: bool) -> None:
    _check(load().lstm_set_profiling(handle, int(bool(enable))), handle)


def lstm_get_profile(handle):
    """Returns dict(proj_us, proj_launches, rec_us, rec_launches) accumulated since the previous call."""
    pu, ru = ctypes.c_double(), ctypes.c_double()
    pn, rn = ctypes.c_int(), ctypes.c_int()
    _check(load().lstm_get_profile(handle, ctypes.byref(pu), ctypes.byref(pn), ctypes.byref(ru), ctypes.byref(rn)), handle)
    return dict(proj_us=pu.value, proj_launches=pn.value, rec_us=ru.value, rec_launches=rn.value)


def lstm_describe_plan(handle) -> str:
    buf = ctypes.create_string_buffer(2048)
    _check(load().lstm_describe_plan(handle, buf, len(buf)), handle)
    return buf.value.decode()


def lstm_get_compressed(handle, layer: int, direction: int, which: int, rows: int):
    lib = load()
    nnz = ctypes.c_int64()
    _check(lib.lstm_get_compressed(handle, layer, direction, which, ctypes.byref(nnz), None, None, None), handle)
    row_ptr = np.zeros(rows + 1, np.int64)
    col = np.zeros(max(nnz.value, 1), np.int32)
    val = np.zeros(max(nnz.value, 1), np.float32)
    _check(lib.lstm_get_compressed(handle, layer, direction, which, ctypes.byref(nnz), row_ptr.ctypes.data,
                                   col.ctypes.data, val.ctypes.data), handle)
    return row_ptr, col[:nnz.value], val[:nnz.value]


def lstm_is_compressed(handle, layer: int, direction: int, which: int) -> bool:
    """True when that matrix is held in row-compressed form (asks lstm_get_compressed for the count only)."""
    nnz = ctypes.c_int64()
    rc = load().lstm_get_compressed(handle, layer, direction, which, ctypes.byref(nnz), None, None, None)
    if rc == LSTM_OK:
        return True
    if rc == LSTM_ERR_STATE:
        return False
    raise LstmError(rc, _err(handle))


def lstm_latency_sweep(Hs: Sequence[int], T: int, B: int, dtype: int = LSTM_F32, seed: int = 1, warmup: int = 10,
                       iters: int = 100, stream: Optional[int] = None):
    Hs = np.ascontiguousarray(Hs, dtype=np.int32)
    n = len(Hs)
    med, p10, p90 = np.zeros(n), np.zeros(n), np.zeros(n)
    flags = np.zeros(n, np.uint8)
    _check(load().lstm_latency_sweep(Hs.ctypes.data, n, T, B, dtype, seed, warmup, iters, med.ctypes.data,
                                     p10.ctypes.data, p90.ctypes.data, flags.ctypes.data, stream))
    return med, p10, p90, flags


def lstm_latency_sweep_model(Hs: Sequence[int], Ds: Optional[Sequence[int]] = None, *, layers: int = 1,
                             bidirectional: bool = False, gate_hidden: bool = False, keep: float = 0.0, T: int = 35,
                             B: int = 1, dtype: int = LSTM_F32, seed: int = 1, warmup: int = 10, iters: int = 100,
                             stream: Optional[int] = None):
    Hs = np.ascontiguousarray(Hs, dtype=np.int32)
    n = len(Hs)
    if Ds is not None:
        Ds = np.ascontiguousarray(Ds, dtype=np.int32)
        assert len(Ds) == n
    med, p10, p90 = np.zeros(n), np.zeros(n), np.zeros(n)
    flags = np.zeros(n, np.uint8)
    _check(load().lstm_latency_sweep_model(Hs.ctypes.data, None if Ds is None else Ds.ctypes.data, n, layers,
                                           int(bool(bidirectional)), int(bool(gate_hidden)), float(keep), T, B, dtype,
                                           seed, warmup, iters, med.ctypes.data, p10.ctypes.data, p90.ctypes.data,
                                           flags.ctypes.data, stream))
    return med, p10, p90, flags


def lstm_grow_to_lhp(dims: Sequence[int], lat: Sequence[float], from_dim: int, eps: float = 0.0):
    dims = np.ascontiguousarray(dims, dtype=np.int32)
    lat = np.ascontiguousarray(lat, dtype=np.float64)
    target = ctypes.c_int()
    gain = ctypes.c_double()
    _check(load().lstm_grow_to_lhp(dims.ctypes.data, lat.ctypes.data, len(dims), eps, from_dim, ctypes.byref(target),
                                   ctypes.byref(gain)))
    return target.value, gain.value


def lstm_find_lhp(dims: Sequence[int], lat: Sequence[float], eps: float = 0.0):
    dims = np.ascontiguousarray(dims, dtype=np.int32)
    lat = np.ascontiguousarray(lat, dtype=np.float64)
    flags = np.zeros(len(dims), np.uint8)
    red = ctypes.c_double()
    _check(load().lstm_find_lhp(dims.ctypes.data, lat.ctypes.data, len(dims), eps, flags.ctypes.data, ctypes.byref(red)))
    return flags, red.value


def lstm_bench_copy(dst_ptr: int, src_ptr: int, nbytes: int, iters: int = 20, stream: Optional[int] = None) -> float:
    us = ctypes.c_double()
    _check(load().lstm_bench_copy(dst_ptr, src_ptr, nbytes, iters, ctypes.byref(us), stream))
    return us.value


def lstm_prune_weights(W_ptr: int, mask_ptr: int, count: int, p_w: float, stream: Optional[int] = None):
    """Device pointers; returns (active before, active after)."""
    before, after = ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().lstm_prune_weights(W_ptr, mask_ptr, count, float(p_w), ctypes.byref(before), ctypes.byref(after), stream))
    return before.value, after.value


def lstm_prune_rows_cols(W_ptr: int, mask_ptr: int, M: int, N: int, p_r: float, p_c: float, stream: Optional[int] = None):
    """Device pointers; returns (rows removed, columns removed)."""
    r, cc = ctypes.c_int(), ctypes.c_int()
    _check(load().lstm_prune_rows_cols(W_ptr, mask_ptr, M, N, float(p_r), float(p_c), ctypes.byref(r), ctypes.byref(cc), stream))
    return r.value, cc.value


def lstm_prune_rows_cols_static(W_ptr: int, mask_ptr: int, M: int, N: int, p_r: float, p_c: float,
                                removed_ptr: Optional[int] = None, stream: Optional[int] = None) -> None:
    """Allocation-free, asynchronous variant; removed_ptr: device int[2] or None."""
    _check(load().lstm_prune_rows_cols_static(W_ptr, mask_ptr, M, N, float(p_r), float(p_c), removed_ptr, stream))


def lstm_compact_rows_cols(W_ptr: int, mask_ptr: int, gates: int, R: int, N: int, row_index_ptr: int, col_index_ptr: int,
                           Wc_ptr: int, mask_c_ptr: Optional[int], stream: Optional[int] = None):
    """Device pointers; returns (units kept, columns kept)."""
    rc, nc = ctypes.c_int(), ctypes.c_int()
    _check(load().lstm_compact_rows_cols(W_ptr, mask_ptr, gates, R, N, row_index_ptr, col_index_ptr, Wc_ptr, mask_c_ptr,
                                         ctypes.byref(rc), ctypes.byref(nc), stream))
    return rc.value, nc.value


def lstm_bench_matmul(n: int, batch: int, keep: float, fmt: int, seed: int = 1, iters: int = 20, want_product: bool = False,
                      stream: Optional[int] = None, X: Optional[np.ndarray] = None, W: Optional[np.ndarray] = None,
                      mask: Optional[np.ndarray] = None):
    """X [batch, n], W [n, n] fp32 and mask [n, n] uint8 (host arrays) replace the library's seeded operands when given."""
    us = ctypes.c_double()
    y = np.zeros((batch, n), np.float32) if want_product else None
    Xc = None if X is None else np.ascontiguousarray(X, np.float32)
    Wc = None if W is None else np.ascontiguousarray(W, np.float32)
    mc = None if mask is None else np.ascontiguousarray(mask, np.uint8)
    for a, shape in ((Xc, (batch, n)), (Wc, (n, n)), (mc, (n, n))):
        if a is not None and a.shape != shape:
            raise ValueError(f"lstm_bench_matmul: operand of shape {a.shape}, expected {shape}")
    _check(load().lstm_bench_matmul(n, batch, float(keep), fmt, seed, iters,
                                    None if Xc is None else Xc.ctypes.data, None if Wc is None else Wc.ctypes.data,
                                    None if mc is None else mc.ctypes.data, ctypes.byref(us),
                                    None if y is None else y.ctypes.data, stream))
    return (us.value, y) if want_product else us.value


def lstm_bench_mfma(dtype: int, reps: int = 20000, iters: int = 3, stream: Optional[int] = None, random_operands: bool = False,
                    with_clock: bool = False):
    """Matrix-instruction issue rate in TFLOP/s (operands in registers); with_clock: (TFLOP/s, shader clock in GHz)."""
    t, g = ctypes.c_double(), ctypes.c_double()
    _check(load().lstm_bench_mfma(dtype, int(bool(random_operands)), reps, iters, ctypes.byref(t), ctypes.byref(g), stream))
    return (t.value, g.value) if with_clock else t.value


def lstm_bench_barrier(workgroups: int, waves: int, steps: int = 200, iters: int = 5, cooperative: bool = True,
                       stream: Optional[int] = None) -> float:
    """Microseconds per round of a device-wide barrier that carries no data."""
    us = ctypes.c_double()
    _check(load().lstm_bench_barrier(workgroups, waves, steps, iters, int(bool(cooperative)), ctypes.byref(us), stream))
    return us.value


def lstm_bench_group_exchange(slots: int, members: int, groups: int, placed: bool, workgroup_stores: bool, steps: int = 200,
                              iters: int = 5, cooperative: bool = True, stream: Optional[int] = None):
    """Returns (microseconds per round, groups whose one-XCD check succeeded)."""
    us, ver = ctypes.c_double(), ctypes.c_int()
    _check(load().lstm_bench_group_exchange(slots, members, groups, int(bool(placed)), int(bool(workgroup_stores)), steps, iters,
                                            int(bool(cooperative)), ctypes.byref(us), ctypes.byref(ver), stream))
    return us.value, ver.value


def lstm_bench_exchange(hidden: int, waves: int = 0, steps: int = 200, iters: int = 5, stream: Optional[int] = None,
                        cooperative: bool = True) -> float:
    us = ctypes.c_double()
    _check(load().lstm_bench_exchange(hidden, waves, steps, iters, int(bool(cooperative)), ctypes.byref(us), stream))
    return us.value


# ------------------------------------------------------------------------------------------------------------
# Convenience wrapper for tests and the benchmark: owns a handle plus torch device buffers.
# ------------------------------------------------------------------------------------------------------------
class Lstm:
    """hidden (and gate_hidden) may be one width for all layers or one per layer.  With per-layer widths the states are
    flat tensors: block n = l * ndir + d holds [B, hidden[l]] values, the blocks follow each other in that order."""

    def __init__(self, layers: int, input_dim: int, hidden, bidirectional: bool = False, dtype: int = LSTM_F32,
                 gate_hidden=0):
        self.layers, self.input_dim = layers, input_dim
        self.ndir = 2 if bidirectional else 1
        self.dtype = dtype
        self.per_layer = not np.isscalar(hidden)
        if self.per_layer:
            self.hiddens = [int(h) for h in hidden]
            assert len(self.hiddens) == layers
            gl = None
            if not np.isscalar(gate_hidden):
                gl = [int(g) for g in gate_hidden]
            elif gate_hidden > 0:
                gl = [int(gate_hidden)] * layers
            self.gate_hidden = 0 if gl is None else max(gl)
            self.hidden = self.hiddens[-1]
            self.handle = lstm_create_layers(input_dim, self.hiddens, gl, bidirectional, dtype)
        else:
            self.hidden = hidden
            self.hiddens = [hidden] * layers
            self.gate_hidden = gate_hidden
            if gate_hidden > 0:
                self.handle = lstm_create_h(layers, input_dim, hidden, gate_hidden, bidirectional, dtype)
            else:
                self.handle = lstm_create(layers, input_dim, hidden, bidirectional, dtype)
        self._ws = None

    def close(self):
        if self.handle is not None:
            lstm_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_weights_from(self, weights, fmt: int = LSTM_FMT_AUTO):
        for (l, d), p in weights.items():
            if self.gate_hidden > 0:
                lstm_set_weights_h(self.handle, l, d, p["W1x"], p.get("M1x"), p["W1h"], p.get("M1h"), p["b1"],
                                   p["W2"], p.get("M2"), p["b2"], fmt)
            else:
                lstm_set_weights(self.handle, l, d, p["Wx"], p.get("Mx"), p["Wh"], p.get("Mh"), p["b"], fmt)

    def forward(self, x, h0=None, c0=None, want_state: bool = True, stream=None, check: bool = True):
        """x: torch device tensor [T,B,D0] (float32, or bfloat16 for bf16 models).  Returns (y, hT, cT)."""
        import torch
        T, B, D0 = x.shape
        assert D0 == self.input_dim and x.is_contiguous()
        assert x.dtype == (torch.bfloat16 if self.dtype == LSTM_BF16 else torch.float32)
        dev = x.device
        n = self.layers * self.ndir
        y = torch.empty((T, B, self.ndir * self.hidden), dtype=torch.float32, device=dev)
        if self.per_layer:
            units = sum(self.hiddens) * self.ndir
            hT = torch.empty(B * units, dtype=torch.float32, device=dev) if want_state else None
            cT = torch.empty(B * units, dtype=torch.float32, device=dev) if want_state else None
        else:
            hT = torch.empty((n, B, self.hidden), dtype=torch.float32, device=dev) if want_state else None
            cT = torch.empty((n, B, self.hidden), dtype=torch.float32, device=dev) if want_state else None
        need = lstm_workspace_bytes(self.handle, T, B)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=dev)
        if stream is None:
            stream = torch.cuda.current_stream(dev).cuda_stream
        lstm_forward(self.handle, T, B, x.data_ptr(),
                     None if h0 is None else h0.data_ptr(), None if c0 is None else c0.data_ptr(),
                     y.data_ptr(), None if hT is None else hT.data_ptr(), None if cT is None else cT.data_ptr(),
                     self._ws.data_ptr(), self._ws.numel(), stream)
        if check:
            torch.cuda.synchronize(dev)
            lstm_check(self.handle)
        return y, hT, cT
