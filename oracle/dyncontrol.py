"""Measured-time batch-size controller: procedure getBsz of Algorithm 1 with its stability
kit (test infrastructure).

Follows section "Proportional Control based Dynamic-Batching" (equations itrtimeerror,
dynbszadjust), section "Control Stability for Dynamic-Batching" (dead-banding, equation
omnibszdeadbandlimit; exponential smoothing; batch-size bounds; the fixed-global-batch
rule, equation dynbszGlobalBFixed) and procedure getBsz of Algorithm 1.  Workers report
the time one iteration took; the controller smooths it, and at the end of an epoch
proposes b* = b - T (t - t_avg) with T = b / t, accepts it only when it differs enough
from the current batch size, and clamps it to the bounds.

The paper computes with real numbers and says nothing of rounding; everything here is
IEEE double arithmetic written one operation per statement so that another
implementation can follow it operation for operation, and integers are made as follows.

Readings (the paper is silent or at odds with itself):
  * smoothing applies to the compute TIME (Algorithm 1), not to the error tau (the prose);
    newest sample weight alpha: ewma = alpha * t + (1 - alpha) * ewma, first sample as is;
    the average restarts after every adjustment (times measured at the old batch size say
    nothing about the new one);
  * the dead-band ratio divides by the NEW batch size, as printed; a worker whose change
    is below the threshold keeps its batch size ("no batch re-adjustments are made");
  * without a global rule each worker decides for itself and the accepted b* is rounded to
    the nearest integer (ties to even) after clamping; the global batch may drift;
  * with the global batch fixed, per-worker decisions cannot keep sum(b) = B, so the
    dead-band is all-or-nothing (everyone moves if any worker's ratio reaches the
    threshold); "proportionately reducing adjusted batches (from Equation dynpropctrl)" is
    read multiplicatively and applied to the unclamped b*: they are turned into integer
    weights (floor(b* * 2^20)) and apportioned over B by largest remainder within the
    bounds (the stateless controller's routine);
  * the printed (subtractive) form of the rule is kept as a non-default variant: every b*
    loses the equal share (sum(b*) - B) / K, is then clamped and rounded; it keeps
    sum(b) = B only up to rounding and only while no clamp fires.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

from .controller import apportion, offsets

RULE_NONE, RULE_MULTIPLICATIVE, RULE_ADDITIVE = 0, 1, 2
WEIGHT_SCALE = float(1 << 20)


class DynController:
    def __init__(self, K: int, B: int, b_min: int = 1, b_max: Optional[int] = None, deadband: float = 0.0,
                 alpha: float = 1.0, global_rule: int = RULE_MULTIPLICATIVE,
                 b_init: Optional[Sequence[int]] = None):
        if b_max is None:
            b_max = B
        if K < 1 or B < K or b_min < 1 or b_max < b_min or not (0.0 <= deadband < 1.0) or not (0.0 < alpha <= 1.0):
            raise ValueError("bad controller arguments")
        if global_rule not in (RULE_NONE, RULE_MULTIPLICATIVE, RULE_ADDITIVE):
            raise ValueError("bad global rule")
        self.K, self.B, self.b_min, self.b_max = K, B, b_min, b_max
        self.deadband, self.alpha, self.rule = float(deadband), float(alpha), global_rule
        # Algorithm 1 starts every worker at B / K (equal shares made integer by largest remainder)
        self.b: List[int] = list(b_init) if b_init is not None else apportion([1] * K, B, 1, B)
        if len(self.b) != K or any(x < 1 for x in self.b):
            raise ValueError("bad initial batch sizes")
        self.ewma: List[float] = [0.0] * K
        self.nobs = 0

    def observe(self, t: Sequence[float]) -> None:
        """One iteration's compute time of every worker (any common unit, > 0)."""
        if len(t) != self.K or any(not (x > 0.0) or x == float("inf") for x in t):
            raise ValueError("compute times must be positive and finite")
        for k in range(self.K):
            x = float(t[k])
            if self.nobs == 0:
                self.ewma[k] = x
            else:
                new_part = self.alpha * x
                old_part = (1.0 - self.alpha) * self.ewma[k]
                self.ewma[k] = new_part + old_part
        self.nobs += 1

    def proposal(self) -> Tuple[List[float], List[float]]:
        """(b*, dead-band ratio) of every worker from the smoothed times."""
        K = self.K
        s = 0.0
        for k in range(K):
            s = s + self.ewma[k]
        t_avg = s / float(K)
        b_star, ratio = [], []
        for k in range(K):
            bk = float(self.b[k])
            T = bk / self.ewma[k]
            tau = self.ewma[k] - t_avg
            delta = T * tau
            bs = bk - delta
            b_star.append(bs)
            ratio.append(abs((bs - bk) / bs))
        return b_star, ratio

    def adjust(self) -> Tuple[List[int], List[int], bool]:
        """End of an epoch: new batch sizes, their offsets, and whether anything changed."""
        if self.nobs == 0:
            raise ValueError("adjust before any observation")
        b_star, ratio = self.proposal()
        lo, hi = float(self.b_min), float(self.b_max)
        old = list(self.b)
        if self.rule == RULE_NONE:
            for k in range(self.K):
                if ratio[k] >= self.deadband:
                    c = min(max(b_star[k], lo), hi)
                    self.b[k] = int(round(c))          # nearest, ties to even
        elif max(ratio) >= self.deadband:
            # the rule acts on the adjusted batches of equation dynbszadjust; the bounds come after it
            if self.rule == RULE_MULTIPLICATIVE:
                w = [max(1, int(x * WEIGHT_SCALE)) for x in b_star]     # floor: the values are positive
                self.b = apportion(w, self.B, self.b_min, self.b_max)
            else:
                s = 0.0
                for x in b_star:
                    s = s + x
                share = (s - float(self.B)) / float(self.K)
                self.b = [int(round(min(max(x - share, lo), hi))) for x in b_star]
        self.nobs = 0
        return list(self.b), offsets(self.b), self.b != old
