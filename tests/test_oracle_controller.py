"""Pins for the controller oracle (CPU only)."""
import itertools
import os
import random
from fractions import Fraction

import pytest

from oracle import controller as C

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hl_table_batches.txt")


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, cores, real, ints = [f.strip() for f in line.split("|")]
        rows.append((name, [int(c) for c in cores.split()], [Fraction(r) for r in real.split()],
                     [int(i) for i in ints.split()]))
    return rows


@pytest.mark.parametrize("name,cores,real,ints", _golden_rows())
def test_hl_table_through_variable_batching_equation(name, cores, real, ints):
    # closed form of equation varbszBSP, evaluated here independently of the oracle
    S = sum(cores)
    assert [Fraction(c * 128, S) for c in cores] == real
    b, off = C.controller_run(cores, 128)
    assert b == ints
    assert off == [0] + list(itertools.accumulate(ints))


def test_benchmark_ratio_1_2_4_8():
    b, off = C.controller_run([1, 2, 4, 8], 480)
    assert b == [32, 64, 128, 256]
    assert off == [0, 32, 96, 224, 480]
    assert C.controller_run([1000, 3000], 32) == ([8, 24], [0, 8, 32])


def test_uniform_throughput_gives_uniform_batches():
    # Algorithm 1 starts every worker at B/K; equal speeds must leave it there.
    for K, B in [(4, 128), (8, 1024), (16, 2048), (3, 33)]:
        b, _ = C.controller_run([777] * K, B)
        assert b == [B // K] * K


def test_proportional_update_closed_form():
    # b - T*tau == T * mean(t): expand the paper's equations by hand.
    rnd = random.Random(1)
    for _ in range(200):
        K = rnd.randint(1, 7)
        b = [Fraction(rnd.randint(1, 200)) for _ in range(K)]
        t = [Fraction(rnd.randint(1, 1000), rnd.randint(1, 1000)) for _ in range(K)]
        new = C.proportional_update(b, t)
        tbar = sum(t) / K
        for k in range(K):
            assert new[k] == (b[k] / t[k]) * tbar
        # slower than average shrinks, faster grows
        for k in range(K):
            if t[k] > tbar:
                assert new[k] < b[k]
            elif t[k] < tbar:
                assert new[k] > b[k]
        # after the fixed-global-batch rule the result depends on throughput only
        B = rnd.randint(K, 500)
        fixed = C.global_batch_rule(new, B)
        Tk = [b[k] / t[k] for k in range(K)]
        assert sum(fixed) == B
        for k in range(K):
            assert fixed[k] == B * Tk[k] / sum(Tk)


def test_independent_of_initial_batch():
    # "works with any initial batch-size": two different starting points, same T.
    T = [Fraction(3), Fraction(5), Fraction(11)]
    outs = []
    for b0 in ([10, 10, 10], [1, 50, 7]):
        b0 = [Fraction(x) for x in b0]
        t = [b0[k] / T[k] for k in range(3)]
        outs.append(C.global_batch_rule(C.proportional_update(b0, t), 60))
    assert outs[0] == outs[1]


def test_brute_force_small_unbounded():
    # every small case: sum, quota, monotonicity, and optimality of largest remainder
    for K in range(1, 5):
        for B in range(K, 13):
            for T in itertools.product(range(1, 6), repeat=K):
                b = C.apportion(T, B, 1, B) if all(
                    (B * t) // sum(T) >= 1 for t in T) else None
                if b is None:
                    continue
                S = sum(T)
                assert sum(b) == B
                for k in range(K):
                    assert abs(Fraction(b[k]) - Fraction(B * T[k], S)) < 1
                for i in range(K):
                    for j in range(K):
                        if T[i] > T[j]:
                            assert b[i] >= b[j]
                        if T[i] == T[j] and i < j:
                            assert b[i] >= b[j]          # ties favour the lower index


def test_largest_remainder_minimises_error_small():
    # Hamilton's method minimises sum |b_k - quota_k| over integer vectors with the right sum.
    for K, B in [(3, 7), (3, 10), (4, 9)]:
        for T in itertools.product(range(1, 5), repeat=K):
            S = sum(T)
            q = [Fraction(B * t, S) for t in T]
            got = C._largest_remainder(list(T), B)
            err = sum(abs(g - x) for g, x in zip(got, q))
            best = min(sum(abs(c - x) for c, x in zip(cand, q))
                       for cand in itertools.product(range(B + 1), repeat=K) if sum(cand) == B)
            assert err == best


def test_scale_invariance_and_large_values():
    T = [1234, 5678, 91011, 1213]
    b1 = C.apportion(T, 2048)
    b2 = C.apportion([t * 10**12 for t in T], 2048)
    assert b1 == b2
    big = [2**63 - 1, 2**62, 2**61 + 12345]
    b = C.apportion(big, 2**31 - 1)
    assert sum(b) == 2**31 - 1


def test_bounds_brute_force():
    rnd = random.Random(7)
    for _ in range(3000):
        K = rnd.randint(1, 5)
        B = rnd.randint(K, 40)
        T = [rnd.randint(1, 30) for _ in range(K)]
        lo = rnd.randint(1, 6)
        hi = rnd.randint(lo, 20)
        feasible = K * lo <= B <= K * hi
        try:
            b = C.apportion(T, B, lo, hi)
        except C.InfeasibleError:
            assert not feasible, (T, B, lo, hi)
            continue
        assert feasible
        assert sum(b) == B and all(lo <= x <= hi for x in b)
        # workers that are not clamped keep the throughput order
        for i in range(K):
            for j in range(K):
                if T[i] > T[j]:
                    assert b[i] >= b[j], (T, B, lo, hi, b)


def test_bad_arguments():
    with pytest.raises(ValueError):
        C.apportion([1, 0], 8)
    with pytest.raises(ValueError):
        C.apportion([], 8)
    with pytest.raises(C.InfeasibleError):
        C.apportion([1, 1, 1], 2)
    with pytest.raises(C.InfeasibleError):
        C.apportion([1, 1], 10, 1, 4)
