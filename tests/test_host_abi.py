"""Host-side checks that need no GPU: the shared library loads and exports every symbol the header
declares, argument errors are reported as codes, and the latency-hysteresis finder agrees with the oracle's
definition on synthetic curves."""
import os
import re

import numpy as np
import pytest

from oracle import lhp as olhp
from paper_1901_10997_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "lstm355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lstm_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    declared = _declared_symbols()
    assert declared, "no declarations parsed"
    assert sorted(B.EXPORTS) == declared
    for name in declared:
        assert hasattr(lib, name), name


def test_create_argument_errors():
    import ctypes
    lib = B.load()
    for args in [(0, 4, 4, 0, 0), (1, 0, 4, 0, 0), (1, 4, 0, 0, 0), (1, 4, 4, 2, 0), (1, 4, 4, 0, 7)]:
        h = ctypes.c_void_p()
        assert lib.lstm_create(*args, ctypes.byref(h)) == B.LSTM_ERR_ARG
        assert not h.value
        assert lib.lstm_last_error(None)
    with pytest.raises(B.LstmError) as ei:
        B.lstm_create(0, 4, 4, False)
    assert ei.value.code == B.LSTM_ERR_ARG
    assert lib.lstm_create(1, 4, 4, 0, 0, None) == B.LSTM_ERR_ARG
    assert lib.lstm_destroy(None) == B.LSTM_OK
    assert lib.lstm_forward(None, 1, 1, None, None, None, None, None, None, None, 0, None) == B.LSTM_ERR_ARG
    assert lib.lstm_set_weights(None, 0, 0, None, None, None, None, None, 0) == B.LSTM_ERR_ARG
    assert lib.lstm_workspace_bytes(None, 1, 1) == 0
    assert lib.lstm_check(None) == B.LSTM_ERR_ARG
    assert lib.lstm_set_plan(None, 0, 0) == B.LSTM_ERR_ARG


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("eps", [0.0, 0.02])
def test_lhp_finder_matches_definition(seed, eps):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    dims = rng.permutation(np.arange(64, 64 + 32 * n, 32)).astype(np.int32)
    # globally increasing, locally non-monotonic: steps plus noise
    lat = 5.0 + 0.01 * dims + 3.0 * np.floor(dims / 256.0) + rng.normal(0, 0.5, n)
    if seed == 3 and n > 2:
        lat[1] = lat[0]          # exact ties
    flags, red = B.lstm_find_lhp(dims, lat, eps)
    ref_flags, ref_red = olhp.find_lhp(list(dims), list(lat), eps)
    assert list(flags) == ref_flags
    assert abs(red - ref_red) < 1e-12
    assert flags[np.argmax(dims)] == 1


def test_lhp_hand_example():
    # staircase: 64..128 cost 10, 160..256 cost 20 except 192 which is slower than 256
    dims = [64, 96, 128, 160, 192, 224, 256]
    lat = [10.0, 10.0, 10.0, 20.0, 21.0, 20.0, 20.0]
    flags, red = B.lstm_find_lhp(dims, lat, 0.0)
    # 256 always; 128 is the first below the 20-plateau; 64/96 tie with 128 (not strictly faster)
    assert list(flags) == [0, 0, 1, 0, 0, 0, 1]
    assert abs(red - (1 - 2 / 7) * 100) < 1e-12
    with pytest.raises(B.LstmError):
        B.lstm_find_lhp(dims, lat, 1.5)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
@pytest.mark.parametrize("eps", [0.0, 0.03])
def test_grow_to_lhp_matches_definition(seed, eps):
    rng = np.random.default_rng(50 + seed)
    n = 40
    dims = rng.permutation(np.arange(64, 64 + 8 * n, 8)).astype(np.int32)
    lat = 20.0 + 0.01 * dims + rng.choice([0.0, 0.5, 2.0], size=n) + rng.uniform(0, 0.3, n)
    for from_dim in (int(dims.min()) - 3, int(np.sort(dims)[n // 2]), int(np.sort(dims)[n // 2]) + 1, int(dims.max())):
        target, gain = B.lstm_grow_to_lhp(dims, lat, from_dim, eps)
        ref_target, ref_gain = olhp.grow_to_lhp(list(dims), list(lat), from_dim, eps)
        assert target == ref_target
        assert abs(gain - ref_gain) < 1e-9
        assert target >= from_dim
        if eps == 0.0:
            assert gain >= -1e-12      # the target is faster than everything above it, the reference included
    with pytest.raises(B.LstmError):
        B.lstm_grow_to_lhp(dims, lat, int(dims.max()) + 1, eps)


def test_grow_to_lhp_hand_example():
    """A staircase: 1197 sits on the same tier as 1200 (cost set by the tier), so growing to 1200 costs nothing and the
    target of everything in (1168, 1200] is 1200; a point that is itself a hysteresis point stays where it is."""
    dims = [1136, 1168, 1197, 1200, 1232, 1264]
    lat = [70.0, 70.1, 75.2, 75.0, 75.1, 80.0]
    assert B.lstm_grow_to_lhp(dims, lat, 1197)[0] == 1200
    t, gain = B.lstm_grow_to_lhp(dims, lat, 1197)
    assert abs(gain - (1 - 75.0 / 75.2) * 100) < 1e-9
    assert B.lstm_grow_to_lhp(dims, lat, 1169)[0] == 1200
    assert B.lstm_grow_to_lhp(dims, lat, 1168) == (1168, 0.0)
    assert B.lstm_grow_to_lhp(dims, lat, 1201)[0] == 1232    # only larger dimensions count: 1232 beats 1264
