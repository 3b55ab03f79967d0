"""Pins for the measured-time controller oracle (procedure getBsz with its stability kit)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import controller as OC
from oracle import dyncontrol as OD


def _times(b, T):
    return [bk / Tk for bk, Tk in zip(b, T)]


def test_proposal_is_the_proportional_update():
    # b - T (t - t_avg) with T = b / t: the exact-rational routine of the stateless oracle, and the closed form b t_avg / t
    rng = np.random.default_rng(0)
    for _ in range(50):
        K = int(rng.integers(2, 9))
        b = [int(x) for x in rng.integers(1, 200, K)]
        t = [float(x) for x in rng.uniform(0.1, 5.0, K)]
        c = OD.DynController(K, sum(b), b_init=b, global_rule=OD.RULE_NONE)
        c.observe(t)
        b_star, _ = c.proposal()
        exact = OC.proportional_update([Fraction(x) for x in b], [Fraction(x) for x in t])
        t_avg = sum(t) / K
        for k in range(K):
            assert b_star[k] == pytest.approx(float(exact[k]), rel=1e-12)
            assert b_star[k] == pytest.approx(b[k] * t_avg / t[k], rel=1e-12)


def test_one_adjustment_reaches_the_throughput_shares():
    # exact times t = b / T, global batch fixed: one step from the uniform start lands on B T_k / sum(T),
    # the allocation of the (separately pinned) stateless controller
    for T, B in (((1000, 2000, 4000, 8000), 480), ((1000, 3000), 32), ((12, 12, 8, 16), 128), ((6, 6, 4, 32), 128)):
        c = OD.DynController(len(T), B)
        c.observe(_times(c.b, T))
        b, off, changed = c.adjust()
        assert b == OC.apportion(list(T), B) and off == OC.offsets(b) and sum(b) == B
    assert OD.DynController(4, 480).b == [120] * 4


def test_deadband_and_bounds():
    # worker 1 is 10 % slow: proposal changes by less than 15 % -> nothing moves; at 5 % threshold it does
    b0 = [32, 32, 32, 32]
    t = [1.0, 1.1, 1.0, 1.0]
    c = OD.DynController(4, 128, deadband=0.15, global_rule=OD.RULE_NONE, b_init=b0)
    c.observe(t)
    assert c.adjust()[0] == b0
    c = OD.DynController(4, 128, deadband=0.05, global_rule=OD.RULE_NONE, b_init=b0)
    c.observe(t)
    b, _, changed = c.adjust()
    t_avg = 4.1 / 4
    assert changed and b[1] == round(32 * t_avg / 1.1) and b[0] == 32      # worker 0 moves 2.5 % only: kept
    # the ratio divides by the NEW batch size: |b* - b| / b*
    c = OD.DynController(2, 64, global_rule=OD.RULE_NONE, b_init=[32, 32])
    c.observe([1.0, 3.0])
    b_star, ratio = c.proposal()
    assert b_star == pytest.approx([64.0, 64.0 / 3]) and ratio == pytest.approx([0.5, 0.5])
    # bounds: HL8 cores (6, 6, 4, 32), bounds (12, 96) as in the paper's static experiment, no global rule
    c = OD.DynController(4, 128, b_min=12, b_max=96, deadband=0.15, global_rule=OD.RULE_NONE)
    c.observe(_times(c.b, (6, 6, 4, 32)))
    b, _, _ = c.adjust()
    assert b[3] == 96 and min(b) >= 12


def test_smoothing_closed_forms():
    c = OD.DynController(1, 8, alpha=0.25)
    for _ in range(5):
        c.observe([2.0])
    assert c.ewma == [2.0]
    # step from 1 to 3: ewma_n = 3 + (1 - 3) (1 - alpha)^n
    c = OD.DynController(1, 8, alpha=0.25)
    c.observe([1.0])
    for n in range(1, 10):
        c.observe([3.0])
        assert c.ewma[0] == pytest.approx(3.0 - 2.0 * 0.75 ** n, rel=1e-12)
    # alpha = 1: no memory; the average restarts after an adjustment
    c = OD.DynController(2, 8, alpha=1.0)
    c.observe([1.0, 5.0]); c.observe([2.0, 2.0])
    assert c.ewma == [2.0, 2.0]
    c.adjust()
    c.observe([7.0, 9.0])
    assert c.ewma == [7.0, 9.0]


def test_subtractive_rule_as_printed():
    # b* = (20, 30, 50, 60), B = 128: Delta B = 32, every worker loses 8
    b0 = [10, 10, 10, 10]
    c = OD.DynController(4, 128, global_rule=OD.RULE_ADDITIVE, b_init=b0)
    # times that make b* = b t_avg / t = (20, 30, 50, 60): t_k = 10 t_avg / b*_k with t_avg the mean of t
    inv = [1 / 20, 1 / 30, 1 / 50, 1 / 60]
    t = [x / (sum(inv) / 4) / 10 * 10 for x in inv]       # t_avg = 1... scaled so that mean(t) * 10 / t_k = b*_k
    t_avg = sum(t) / 4
    t = [x / t_avg for x in t]                              # mean exactly 1 up to rounding
    c.observe(t)
    b_star, _ = c.proposal()
    share = (sum(b_star) - 128) / 4
    b, _, _ = c.adjust()
    assert b == [int(round(x - share)) for x in b_star]
    # the reason it is not the default: from the uniform start at a 1:2:4:8 spread it wants a negative batch
    c = OD.DynController(4, 480, global_rule=OD.RULE_ADDITIVE)
    c.observe(_times(c.b, (1000, 2000, 4000, 8000)))
    b_star, _ = c.proposal()
    assert b_star[0] - (sum(b_star) - 480) / 4 < 0
    assert c.adjust()[0][0] == 1                              # clamped to b_min; the sum is no longer B


def test_settles_within_a_few_adjustments_under_static_heterogeneity():
    # throughput proportional to the cores of the paper's HL table, exact times, 15 % dead-band, bounds (12, 96),
    # no global rule, initial batch 32 everywhere (the static experiment of the evaluation section)
    for cores in ((12, 12, 8, 16), (9, 9, 6, 24), (6, 6, 4, 32)):
        c = OD.DynController(4, 128, b_min=12, b_max=96, deadband=0.15, global_rule=OD.RULE_NONE)
        history = [list(c.b)]
        for epoch in range(12):
            for it in range(3):
                c.observe(_times(c.b, cores))
            b, _, changed = c.adjust()
            history.append(b)
        last_change = max(i for i in range(1, len(history)) if history[i] != history[i - 1])
        assert last_change <= 4, (cores, history)
        t = _times(history[-1], cores)
        free = [k for k in range(4) if 12 < history[-1][k] < 96]
        assert max(t[k] for k in free) / min(t[k] for k in free) < 1.2     # equalised up to the dead-band
    # with the global batch fixed the sum never moves
    c = OD.DynController(4, 128, b_min=4, b_max=96, deadband=0.10)
    for cores in ((12, 12, 12, 12), (12, 12, 8, 16), (9, 9, 6, 24), (6, 6, 4, 32), (12, 12, 12, 12)):
        for epoch in range(3):
            c.observe(_times(c.b, cores))
            b, _, _ = c.adjust()
            assert sum(b) == 128 and min(b) >= 4 and max(b) <= 96
    assert b == [32, 32, 32, 32]
