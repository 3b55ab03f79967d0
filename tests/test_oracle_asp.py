"""Pins for the asynchronous-training oracle (oracle/asp.py): things the paper and the
mathematics fix, none of which restate the oracle's own code.  CPU only."""
import heapq
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import asp
from oracle.controller import apportion
from synth import nets
from synth.data import he_normal_params

# ASP rows of the paper's table "Heterogeneity configurations (CPU-core allocation) across 4 workers"
ASP_CORES = {"HL1": (10, 10, 10, 10), "HL2": (8, 8, 8, 16), "HL4": (10, 10, 4, 16), "HL8": (4, 4, 4, 28)}


def heap_schedule(T, b, n):
    """Independent event simulation: a priority queue of (finish time, worker) with exact
    times; a worker re-enters the queue right after its push."""
    K = len(T)
    h = [(Fraction(b[k], T[k]), k, 0) for k in range(K)]       # (finish, worker, pulled version)
    heapq.heapify(h)
    worker, version = [], []
    for e in range(n):
        t, k, v = heapq.heappop(h)
        worker.append(k)
        version.append(v)
        heapq.heappush(h, (t + Fraction(b[k], T[k]), k, e + 1))
    return worker, version


def test_schedule_against_priority_queue_simulation():
    rng = np.random.default_rng(5)
    for trial in range(200):
        K = int(rng.integers(1, 7))
        T = [int(v) for v in rng.integers(1, 40, size=K)]
        b = [int(v) for v in rng.integers(1, 40, size=K)]
        n = int(rng.integers(0, 60))
        assert asp.schedule(T, b, n) == heap_schedule(T, b, n), (T, b, n)


def pushes_before(t, k, m, T, b):
    """How many pushes of worker m are ordered before a push of worker k at time t
    (simultaneous pushes: lower index first)."""
    q = t * T[m] / b[m]
    return math.floor(q) if m < k else math.ceil(q) - 1


def test_staleness_closed_form():
    """Push e of worker k (its j-th, at time j b_k / T_k) was computed on the model pulled at
    its previous push: staleness = pushes of the OTHER workers between the two."""
    rng = np.random.default_rng(6)
    for trial in range(100):
        K = int(rng.integers(2, 6))
        T = [int(v) for v in rng.integers(1, 30, size=K)]
        b = [int(v) for v in rng.integers(1, 30, size=K)]
        worker, version = asp.schedule(T, b, 80)
        count = [0] * K
        for e, k in enumerate(worker):
            count[k] += 1
            t1 = Fraction(count[k] * b[k], T[k])
            t0 = Fraction((count[k] - 1) * b[k], T[k])
            others = sum(pushes_before(t1, k, m, T, b) - max(pushes_before(t0, k, m, T, b), 0)
                         for m in range(K) if m != k)
            if count[k] == 1:
                others = sum(pushes_before(t1, k, m, T, b) for m in range(K) if m != k)
            assert e - version[e] == others, (T, b, e)
            # and e itself = all pushes ordered before it
            assert e == count[k] - 1 + sum(pushes_before(t1, k, m, T, b) for m in range(K) if m != k)


def test_uniform_workers_round_robin():
    worker, version = asp.schedule([7, 7, 7], [5, 5, 5], 9)
    assert worker == [0, 1, 2, 0, 1, 2, 0, 1, 2]
    assert [e - v for e, v in enumerate(version)] == [0, 1, 2, 2, 2, 2, 2, 2, 2]


@pytest.mark.parametrize("level", list(ASP_CORES))
def test_variable_batching_equalises_updates(level):
    """Section "Variable Batching", asynchronous training: with throughput proportional to
    the cores and equal batches, a worker's share of the updates is its share of the cores
    (the skewed iteration densities of the uniform-batching figures); with batches
    proportional to the cores every iteration takes the same time, every worker pushes
    equally often and every update is exactly K - 1 pushes stale."""
    c = ASP_CORES[level]
    K, n = 4, 4000
    worker, version = asp.schedule(c, [32] * K, n)
    share = np.bincount(worker, minlength=K) / n
    np.testing.assert_allclose(share, np.array(c) / sum(c), atol=1.0 / n * K)
    # batches in the exact ratio of the cores (a multiple of sum(c), so no rounding)
    bv = [ck * 4 for ck in c]
    worker, version = asp.schedule(c, bv, n)
    assert np.bincount(worker, minlength=K).tolist() == [n // K] * K
    assert all(e - version[e] == K - 1 for e in range(K, n))
    # integer batches of the global batch the paper uses (K * 32): durations differ by
    # less than one sample's worth, so the update counts differ by at most a few per thousand
    bi = apportion(list(c), 128)
    worker, _ = asp.schedule(c, bi, n)
    cnt = np.bincount(worker, minlength=K)
    assert cnt.max() - cnt.min() <= 0.1 * n / K


def test_learning_rates():
    """Equation aspvariableSGD: eta_k = eta b_k / sum(b); they add up to eta."""
    b = [16, 16, 11, 85]
    e = [asp.worker_lr(0.1, bk, 128) for bk in b]
    assert abs(sum(e) - 0.1) < 1e-15
    assert e[3] / e[0] == pytest.approx(85 / 16, rel=1e-15)
    assert asp.worker_lr(0.1, 11, 128, lr_scaling=False) == 0.1


def linear_grad(c):
    """A 'loss' whose gradient does not depend on the model: F(s, theta) = <c_s, theta>;
    batch rows ARE the c_s."""
    return lambda th, x, y: (x.mean(axis=0), float(x.mean(axis=0) @ th))


def test_run_model_independent_gradients():
    """If gradients do not depend on the model, staleness cannot matter: the server model is
    theta_0 - sum_e eta_{k_e} mean(rows of push e)."""
    rng = np.random.default_rng(7)
    K, P, B = 3, 5, 12
    b = [2, 4, 6]
    T = [3, 1, 2]
    worker, version = asp.schedule(T, b, 15)
    data = {e: rng.standard_normal((b[k], P)) for e, k in enumerate(worker)}
    th0 = rng.standard_normal(P)
    vs, _ = asp.run(None, th0, lambda e, k: (data[e], None), worker, version, b, B, lr=0.3,
                    grad_fn=linear_grad(None))
    expect = th0.copy()
    for e, k in enumerate(worker):
        expect = expect - 0.3 * b[k] / B * data[e].mean(axis=0)
    np.testing.assert_allclose(vs[-1], expect, rtol=0, atol=1e-14)
    assert len(vs) == 16


def quad_grad(th, x, y):
    """F(s, theta) = 1/2 |theta - s|^2: gradient theta - mean(s)."""
    m = x.mean(axis=0)
    return th - m, float(0.5 * ((th - x) ** 2).sum(axis=1).mean())


def test_run_stale_quadratic_by_hand():
    """Two workers, scalar model, quadratic loss, worked by hand.  T = (2, 1), b = (1, 1):
    pushes in order w0 (t=1/2), w0 (t=1, index 0 before 1), w1 (t=1), w0 (t=3/2), ...
    eta = 1/2, B = 2 => eta_k = 1/4.  Samples: worker 0 always 4, worker 1 always 0."""
    worker, version = asp.schedule([2, 1], [1, 1], 4)
    assert worker == [0, 0, 1, 0]
    assert version == [0, 1, 0, 2]
    s = {0: 4.0, 1: 0.0}
    vs, _ = asp.run(None, np.array([0.0]), lambda e, k: (np.array([[s[k]]]), None), worker, version,
                    [1, 1], 2, lr=0.5, grad_fn=quad_grad)
    # v1 = 0 - 1/4 (0 - 4) = 1;  v2 = 1 - 1/4 (1 - 4) = 7/4
    # push 2 by worker 1, computed at version 0 (theta = 0): g = 0 - 0 = 0 -> v3 = 7/4
    # push 3 by worker 0, pulled version 2 (7/4): g = 7/4 - 4 = -9/4 -> v4 = 7/4 + 9/16 = 37/16
    np.testing.assert_allclose([v[0] for v in vs], [0.0, 1.0, 1.75, 1.75, 37 / 16], atol=1e-15)
    # the printed push (server model replaced): push 2 throws worker 0's progress away
    vo, _ = asp.run(None, np.array([0.0]), lambda e, k: (np.array([[s[k]]]), None), worker, version,
                    [1, 1], 2, lr=0.5, grad_fn=quad_grad, mode="overwrite")
    # v1 = 1, v2 = 7/4, v3 = 0 - 1/4 * 0 = 0 (worker 1's stale local model), v4 = 7/4 + 9/16
    np.testing.assert_allclose([v[0] for v in vo], [0.0, 1.0, 1.75, 0.0, 37 / 16], atol=1e-15)


def test_overwrite_mode_is_private_chains():
    """With the push as printed and an immediate re-pull, worker k only ever sees its own
    pushes: the server model after push e equals worker k_e's private plain-SGD chain."""
    rng = np.random.default_rng(8)
    K, P, B = 3, 4, 9
    b, T = [2, 3, 4], [5, 3, 4]
    worker, version = asp.schedule(T, b, 20)
    data = {e: rng.standard_normal((b[k], P)) for e, k in enumerate(worker)}
    th0 = rng.standard_normal(P)
    vs, _ = asp.run(None, th0, lambda e, k: (data[e], None), worker, version, b, B, lr=0.2,
                    grad_fn=quad_grad, mode="overwrite")
    chain = [th0.copy() for _ in range(K)]
    for e, k in enumerate(worker):
        chain[k] = chain[k] - 0.2 * b[k] / B * (chain[k] - data[e].mean(axis=0))
        np.testing.assert_allclose(vs[e + 1], chain[k], atol=1e-14)


def test_single_worker_is_plain_sgd_against_library_optimiser():
    """K = 1: no staleness, eta_1 = eta; the run is minibatch SGD.  Checked against an
    independent autograd library and its own SGD optimiser on a small network."""
    torch = pytest.importorskip("torch")
    layers = nets.mlp([6, 5, 3])
    P = nets.param_count(layers)
    assert P == 5 * 6 + 5 + 3 * 5 + 3
    th0 = he_normal_params(layers, 3, bf16=False).astype(np.float64)
    th0 += 0.1 * np.random.default_rng(3).standard_normal(P)
    rng = np.random.default_rng(4)
    batches = [(rng.standard_normal((4, 1, 1, 6)), rng.integers(0, 3, size=4)) for _ in range(5)]
    worker, version = asp.schedule([1], [4], 5)
    assert version == [0, 1, 2, 3, 4]
    vs, losses = asp.run(layers, th0, lambda e, k: batches[e], worker, version, [4], 4, lr=0.05)

    l1, l2 = torch.nn.Linear(6, 5).double(), torch.nn.Linear(5, 3).double()
    with torch.no_grad():
        l1.weight.copy_(torch.tensor(th0[0:30].reshape(5, 6)))
        l1.bias.copy_(torch.tensor(th0[30:35]))
        l2.weight.copy_(torch.tensor(th0[35:50].reshape(3, 5)))
        l2.bias.copy_(torch.tensor(th0[50:53]))
    model = torch.nn.Sequential(l1, torch.nn.ReLU(), l2)
    opt = torch.optim.SGD(model.parameters(), lr=0.05)
    for i, (x, y) in enumerate(batches):
        opt.zero_grad()
        loss = torch.nn.functional.cross_entropy(model(torch.tensor(x.reshape(4, 6))), torch.tensor(y))
        loss.backward()
        opt.step()
        assert losses[i] == pytest.approx(loss.item(), rel=1e-12)
        flat = np.concatenate([l1.weight.detach().numpy().ravel(), l1.bias.detach().numpy(),
                               l2.weight.detach().numpy().ravel(), l2.bias.detach().numpy()])
        np.testing.assert_allclose(vs[i + 1], flat, rtol=1e-12, atol=1e-14)


def test_get_bsz_exact_rational():
    """b - T (t - t_avg) = b t_avg / t (equation dynbszadjust with T = b / t): the double
    result rounds to the same integer as the exact rational away from .5 ties."""
    rng = np.random.default_rng(9)
    for _ in range(2000):
        b = int(rng.integers(1, 500))
        t = Fraction(int(rng.integers(1, 1000)), 64)
        ta = Fraction(int(rng.integers(1, 1000)), 64)
        exact = b * ta / t
        if abs((exact - math.floor(exact)) - Fraction(1, 2)) < Fraction(1, 10 ** 6):
            continue
        want = min(max(math.floor(exact + Fraction(1, 2)), 1), 10 ** 6)
        assert asp.get_bsz(b, float(t), float(ta), 0.0, 1, 10 ** 6) == want


def test_get_bsz_deadband_and_bounds():
    # b = 100, t = 1.0, t_avg = 0.9: b* = 90, |90 - 100| / 90 = 0.111
    assert asp.get_bsz(100, 1.0, 0.9, 0.10, 1, 1000) == 90
    assert asp.get_bsz(100, 1.0, 0.9, 0.12, 1, 1000) == 100
    assert asp.get_bsz(100, 1.0, 0.9, 0.0, 95, 1000) == 95
    assert asp.get_bsz(100, 1.0, 3.0, 0.0, 1, 256) == 256


def test_eval_bsz_bookkeeping():
    """Algorithm 2, procedure evalBsz: nothing changes until all K workers have reported;
    from then on every report returns the caller's new size from the latest times."""
    ps = asp.ParameterServer(3, 1, 1000, 0.0)
    assert ps.eval_bsz(0, 30, 1.0) == 30
    assert ps.eval_bsz(2, 30, 4.0) == 30
    # third report: mean time = (1 + 2 + 4) / 3 = 7/3; worker 1: 30 * (7/3) / 2 = 35
    assert ps.eval_bsz(1, 30, 2.0) == 35
    assert ps.wrk_b == {0: 70, 1: 35, 2: 18}            # 30*(7/3)/1, /2, /4 = 70, 35, 17.5 -> 18 (ties to even)
    # worker 0 reports its next epoch with the size it actually used (30): the map entry is replaced
    # times now (1.5, 2, 4): mean 2.5 -> 30 * 2.5 / 1.5 = 50
    assert ps.eval_bsz(0, 30, 1.5) == 50
    with pytest.raises(ValueError):
        ps.eval_bsz(3, 30, 1.0)
    with pytest.raises(ValueError):
        ps.eval_bsz(0, 30, 0.0)


def test_eval_bsz_settles_to_core_shares():
    """Workers whose time per sample is 1 / c_k (the ASP core table): iterating report ->
    new size -> time = b / c reaches b_k proportional to c_k, where all times are equal."""
    for c in ASP_CORES.values():
        ps = asp.ParameterServer(4, 1, 10 ** 6, 0.0)
        b = [3200] * 4
        for epoch in range(30):
            for k in range(4):
                b[k] = ps.eval_bsz(k, b[k], b[k] / c[k])
        t = [b[k] / c[k] for k in range(4)]
        assert max(t) / min(t) < 1.01
