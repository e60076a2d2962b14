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
