"""Oracle for the latency-hysteresis post-processing.  TEST INFRASTRUCTURE ONLY.

Definitions restated from the paper's Section 3: latency falls with the dimension
globally, but locally it can stall or rise as the dimension shrinks; the point at which
such a stretch begins is a latency hysteresis point (LHP), and every smaller dimension
inside the stretch is no faster than its LHP.  Caption of the model-level latency figure:
architecture-space redundancy = (1 - #LHPs / #design points) * 100 %.

Reading used here: a dimension is an LHP iff it is strictly faster (by a relative margin
eps) than every larger dimension in the list; the largest dimension is always one.
"""
from typing import List, Sequence, Tuple


def find_lhp(dims: Sequence[int], lat: Sequence[float], eps: float = 0.0) -> Tuple[List[int], float]:
    n = len(dims)
    flags = []
    for i in range(n):
        ok = True
        for j in range(n):
            if dims[j] > dims[i] and not (lat[i] < (1.0 - eps) * lat[j]):
                ok = False
        flags.append(1 if ok else 0)
    redundancy = (1.0 - sum(flags) / n) * 100.0 if n else 0.0
    return flags, redundancy


def grow_to_lhp(dims: Sequence[int], lat: Sequence[float], from_dim: int, eps: float = 0.0) -> Tuple[int, float]:
    """Growth target of the hardware-guided step (Section 4: the growth algorithm recovers the model back to its
    LHP; Section 5.1 step (c): 1197 -> 1200): the smallest LHP among the measured dimensions that is not below
    from_dim, and the latency reduction (percent) against the smallest measured dimension not below from_dim."""
    flags, _ = find_lhp(dims, lat, eps)
    cands = [(dims[i], lat[i]) for i in range(len(dims)) if flags[i] and dims[i] >= from_dim]
    if not cands:
        raise ValueError("from_dim is above every measured dimension")
    target, tlat = min(cands)
    ref_dim, ref_lat = min((dims[i], lat[i]) for i in range(len(dims)) if dims[i] >= from_dim)
    return target, (1.0 - tlat / ref_lat) * 100.0
