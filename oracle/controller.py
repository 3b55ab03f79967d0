"""Batch-size controller oracle: exact rationals, then exact integers.

Test infrastructure only.  Follows the paper's section "Dynamic-Batching"
(equations itrtimeerror / dynbszadjust), the fixed-global-batch rule of
section "Control Stability for Dynamic-Batching" (equation
dynbszGlobalBFixed and the sentence after it) and the bounds of procedure
getBsz in Algorithm 1.

Readings taken where the paper is silent or at odds with itself:
  * the global-batch rule is applied multiplicatively (the text's
    "proportionately"), not by subtracting an equal share as the printed
    equation does: the subtractive form can produce negative batch sizes;
  * real-valued batch sizes are made integers by largest remainder, ties to
    the lowest worker index, so the sum is exactly B;
  * bounds are enforced by clamping violators and re-apportioning the rest.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Optional, Sequence


class InfeasibleError(ValueError):
    pass


def proportional_update(b: Sequence[Fraction], t: Sequence[Fraction]) -> List[Fraction]:
    """One proportional-control adjustment (equations itrtimeerror, dynbszadjust).

    b[k] is worker k's current batch size and t[k] the time it took to process
    it.  Throughput T_k = b_k / t_k, error tau_k = t_k - mean(t), and the new
    batch size is b_k - T_k * tau_k."""
    K = len(b)
    t_bar = sum(t, Fraction(0)) / K
    out = []
    for k in range(K):
        T_k = Fraction(b[k]) / Fraction(t[k])
        tau_k = Fraction(t[k]) - t_bar
        out.append(Fraction(b[k]) - T_k * tau_k)
    return out


def global_batch_rule(b_star: Sequence[Fraction], B: int) -> List[Fraction]:
    """Keep the global batch fixed at B by scaling every adjusted batch size by
    B / sum(b_star) (multiplicative reading of the fixed-global-batch rule)."""
    s = sum(b_star, Fraction(0))
    return [Fraction(x) * B / s for x in b_star]


def _largest_remainder(weights: Sequence[int], total: int) -> List[int]:
    """Integers q_k summing to `total`, each within 1 of total*w_k/sum(w):
    floor every quota, then hand the left-over units to the largest fractional
    parts, lowest index first among equals."""
    W = sum(weights)
    q = [(total * w) // W for w in weights]
    r = [(total * w) % W for w in weights]
    left = total - sum(q)
    order = sorted(range(len(weights)), key=lambda k: (-r[k], k))
    for k in order[:left]:
        q[k] += 1
    return q


def apportion(T: Sequence[int], B: int, b_min: int = 1, b_max: Optional[int] = None) -> List[int]:
    """Integer batch sizes proportional to integer throughputs T with sum B and
    b_min <= b_k <= b_max.

    Unbounded case: largest remainder on the quotas B*T_k/sum(T).  If some
    worker falls outside the bounds, the side (low or high) with the larger
    total violation is clamped to its bound, those workers and their units
    leave the pool, and the rest is apportioned again."""
    K = len(T)
    if b_max is None:
        b_max = B
    if K < 1 or B < 1 or any(int(t) <= 0 for t in T) or b_min < 1 or b_max < b_min:
        raise ValueError("bad controller arguments")
    if K * b_min > B or K * b_max < B:
        raise InfeasibleError("bounds cannot hold with sum(b) = B")
    b = [0] * K
    active = list(range(K))
    remaining = B
    while True:
        if not active:
            if remaining != 0:
                raise InfeasibleError("clamping left units unassigned")
            return b
        if remaining < 0:
            raise InfeasibleError("clamping over-assigned")
        share = _largest_remainder([int(T[k]) for k in active], remaining)
        low = [(k, s) for k, s in zip(active, share) if s < b_min]
        high = [(k, s) for k, s in zip(active, share) if s > b_max]
        if not low and not high:
            for k, s in zip(active, share):
                b[k] = s
            return b
        deficit = sum(b_min - s for _, s in low)
        excess = sum(s - b_max for _, s in high)
        if excess >= deficit and high:
            fixed = {k: b_max for k, _ in high}
        else:
            fixed = {k: b_min for k, _ in low}
        for k, v in fixed.items():
            b[k] = v
            remaining -= v
        active = [k for k in active if k not in fixed]


def offsets(b: Sequence[int]) -> List[int]:
    """Exclusive prefix sum: where each worker's slice starts in the concatenated batch."""
    off = [0]
    for x in b:
        off.append(off[-1] + int(x))
    return off


def controller_run(T: Sequence[int], B: int, b_min: int = 1, b_max: Optional[int] = None):
    """Throughputs -> (b, off).

    Walks the paper's chain in exact rationals starting from the uniform batch
    B/K of Algorithm 1: with throughput T_k a worker needs t_k = b_k/T_k, the
    proportional update gives b_k - T_k*tau_k, the global rule rescales to sum
    B; the result must equal B*T_k/sum(T) (checked), which is then made
    integer and bounded by `apportion`."""
    K = len(T)
    b0 = [Fraction(B, K)] * K
    t = [b0[k] / Fraction(int(T[k])) for k in range(K)]
    b_real = global_batch_rule(proportional_update(b0, t), B)
    S = sum(int(x) for x in T)
    assert all(b_real[k] == Fraction(B * int(T[k]), S) for k in range(K))
    b = apportion(T, B, b_min, b_max)
    return b, offsets(b)
