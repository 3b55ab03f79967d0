"""Static variable batching and the memory model that caps batch sizes (test infrastructure).

Follows equation varbszBSP (section "Variable Batching": b_k = c_k / sum(c) * K b, c_k the
compute resource of worker k), equation hlevel (heterogeneity level = largest / smallest
resource) and section "Heterogeneous memory across workers" (equation hetmemeqn:
M_total = M_model + M_grad + M_opt + M_act + M_batch, the first three fixed multiples of the
model size, M_act and M_batch linear in the batch size, M_batch fitted by linear regression on
measured points).  Exact rationals wherever the inputs are integers.

Readings: integers are made by the same largest-remainder apportionment as the dynamic
controller; M_opt is opt_copies model-sized buffers (0 plain SGD, 1 momentum, 2 Adam-like);
the batch-size cap is the largest b whose predicted total fits the worker's memory, the
prediction being evaluated in doubles exactly as written in memory_total.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Optional, Sequence, Tuple

from .controller import apportion, offsets


def real_batches(c: Sequence[int], B: int) -> List[Fraction]:
    """Equation varbszBSP with K b = B, as exact fractions."""
    S = sum(int(x) for x in c)
    return [Fraction(int(x) * B, S) for x in c]


def static_batches(c: Sequence[int], B: int, b_min: int = 1, b_max: Optional[int] = None):
    b = apportion([int(x) for x in c], B, b_min, b_max)
    return b, offsets(b)


def heterogeneity_level(c: Sequence[int]) -> Fraction:
    """Equation hlevel."""
    return Fraction(max(c), min(c))


def fit_linear(b: Sequence[int], m: Sequence[int]) -> Tuple[Fraction, Fraction]:
    """Least-squares line m ~ slope * b + intercept through measured (batch size, bytes)
    points, by the normal equations in exact rationals."""
    n = len(b)
    if n < 2 or len(m) != n or len(set(b)) < 2:
        raise ValueError("need at least two distinct batch sizes")
    sb = sum(Fraction(x) for x in b)
    sm = sum(Fraction(x) for x in m)
    sbb = sum(Fraction(x) * x for x in b)
    sbm = sum(Fraction(x) * y for x, y in zip(b, m))
    slope = (n * sbm - sb * sm) / (n * sbb - sb * sb)
    intercept = (sm - slope * sb) / n
    return slope, intercept


def memory_total(b: int, P: int, bytes_per_param: int, opt_copies: int, act_per_sample: float,
                 batch_slope: float, batch_intercept: float) -> float:
    """Equation hetmemeqn in doubles, one operation per statement."""
    model = float(P) * float(bytes_per_param)
    fixed3 = (2.0 + float(opt_copies)) * model          # M_model + M_grad + M_opt
    act = act_per_sample * float(b)
    batch_var = batch_slope * float(b)
    batch = batch_var + batch_intercept
    s1 = fixed3 + act
    return s1 + batch


def max_batch(mem_avail: float, P: int, bytes_per_param: int, opt_copies: int, act_per_sample: float,
              batch_slope: float, batch_intercept: float, limit: int = 1 << 30) -> int:
    """Largest b in [0, limit] with memory_total(b) <= mem_avail; 0 when only the fixed part
    fits, -1 when not even that does."""
    def fits(b):
        return memory_total(b, P, bytes_per_param, opt_copies, act_per_sample, batch_slope, batch_intercept) <= mem_avail
    if not fits(0):
        return -1
    lo, hi = 0, limit
    if fits(hi):
        return hi
    while hi - lo > 1:                 # fits(lo) and not fits(hi); the prediction is non-decreasing in b
        mid = (lo + hi) // 2
        if fits(mid):
            lo = mid
        else:
            hi = mid
    return lo
