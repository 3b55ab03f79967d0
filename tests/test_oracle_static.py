"""Pins for static variable batching, the heterogeneity level and the memory model
(oracle/static.py).  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import static as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hl_table_levels.txt")


def _rows():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            name, cores, hl, total = [f.strip() for f in line.split("|")]
            out.append((name, [int(c) for c in cores.split()], int(hl), int(total)))
    return out


@pytest.mark.parametrize("name,cores,hl,total", _rows())
def test_heterogeneity_levels_of_the_paper(name, cores, hl, total):
    assert S.heterogeneity_level(cores) == hl
    assert sum(cores) == total


@pytest.mark.parametrize("name,cores,hl,total", _rows())
def test_static_batches_properties(name, cores, hl, total):
    """Equation varbszBSP: shares add up to the global batch, are proportional to the cores
    (b_i c_j = b_j c_i) and the largest / smallest share ratio is the heterogeneity level;
    the integers stay within one of the real values."""
    B = 128
    real = S.real_batches(cores, B)
    assert sum(real) == B
    for i in range(4):
        for j in range(4):
            assert real[i] * cores[j] == real[j] * cores[i]
    assert max(real) / min(real) == hl
    b, off = S.static_batches(cores, B)
    assert sum(b) == B and off[-1] == B
    assert all(abs(bi - ri) < 1 for bi, ri in zip(b, real))


def test_static_batches_with_bounds_of_the_experiments():
    # section "Evaluation": b_min = 12, b_max = 96 around an initial batch of 32
    # HL8: real shares 16, 16, 10.67, 85.33; worker 3 is raised to 12, the other 116 samples are
    # shared 6:6:32 -> 15.82, 15.82, 84.36 -> 15, 15, 84 and the two left over go to the .82s
    b, _ = S.static_batches([6, 6, 4, 32], 128, 12, 96)
    assert b == [16, 16, 12, 84]


def test_fit_linear_against_library_and_exact_line():
    rng = np.random.default_rng(3)
    # the batch sizes the paper measured the data loader at
    bs = [1, 32, 64, 128, 512, 1024]
    exact = [3 * 1024 * 32 * 32 * x + 7_000_000 for x in bs]
    slope, icpt = S.fit_linear(bs, exact)
    assert slope == 3 * 1024 * 32 * 32 and icpt == 7_000_000
    for _ in range(20):
        m = [int(150_000 * x + 5e6 + rng.normal(0, 2e5)) for x in bs]
        slope, icpt = S.fit_linear(bs, m)
        ref = np.polyfit(np.array(bs, dtype=np.float64), np.array(m, dtype=np.float64), 1)
        assert float(slope) == pytest.approx(ref[0], rel=1e-9)
        assert float(icpt) == pytest.approx(ref[1], rel=1e-7)
    with pytest.raises(ValueError):
        S.fit_linear([4, 4], [1, 2])


def test_memory_total_terms():
    """Each term of equation hetmemeqn on its own."""
    P = 11_000_000
    base = S.memory_total(0, P, 4, 0, 0.0, 0.0, 0.0)
    assert base == 2 * 4 * P                                        # model + gradients
    assert S.memory_total(0, P, 4, 1, 0.0, 0.0, 0.0) == 3 * 4 * P   # + momentum buffer
    assert S.memory_total(0, P, 2, 2, 0.0, 0.0, 0.0) == 4 * 2 * P   # half precision, two optimiser buffers
    assert S.memory_total(10, P, 4, 0, 1000.0, 0.0, 0.0) - base == 10_000
    assert S.memory_total(10, P, 4, 0, 0.0, 300.0, 50.0) - base == 3050


def test_max_batch_against_linear_scan():
    rng = np.random.default_rng(4)
    for _ in range(300):
        P = int(rng.integers(1, 5000))
        act = float(rng.uniform(1, 500))
        slope = float(rng.uniform(0, 300))
        icpt = float(rng.uniform(0, 5000))
        opt = int(rng.integers(0, 3))
        mem = float(rng.uniform(0, 400_000))
        got = S.max_batch(mem, P, 4, opt, act, slope, icpt, limit=5000)
        scan = -1
        for b in range(0, 5001):
            if S.memory_total(b, P, 4, opt, act, slope, icpt) <= mem:
                scan = b
            else:
                break
        assert got == scan


def test_max_batch_closed_form():
    # 1 GiB worker, 1M-parameter fp32 model with momentum (12 MB fixed), 2 MiB of activations and
    # 0.5 MiB of loader memory per sample, 100 MiB loader overhead:
    # (1024 - 100) MiB - 12e6 B = 956,892,224 B; / 2,621,440 B per sample = 365.02 -> 365
    assert S.max_batch(float(1 << 30), 1_000_000, 4, 1, float(2 << 20), float(1 << 19), float(100 << 20)) == 365
