"""GPU parity of the single-kernel entry points: weighted aggregation + update, softmax cross-entropy."""
import numpy as np
import pytest

from oracle import layers as OL

from gpu_util import assert_close

pytestmark = pytest.mark.gpu


def _oracle_weighted_sgd(theta, G, b, lr):
    """theta - lr * sum_k (b_k / sum b) g_k, k ascending, fp64 (equations bspweightedgrads, bspvariableSGD)."""
    B = float(sum(b))
    g = np.zeros(theta.size)
    for k in range(len(b)):
        g += (b[k] / B) * G[k].astype(np.float64)
    return theta.astype(np.float64) - lr * g, g


@pytest.mark.parametrize("P,K", [(9610, 2), (4206602, 4), (113738, 16), (1, 1), (3, 5), (1027, 64), (11220132, 8)])
def test_weighted_sgd(P, K):
    import torch
    import paper_2503_17469_amd as omni
    print(f"case weighted_sgd P={P} K={K}", flush=True)
    rng = np.random.default_rng(P + K)
    stride = (P + 63) // 64 * 64
    theta = rng.standard_normal(P).astype(np.float32)
    G = np.zeros((K, stride), dtype=np.float32)
    G[:, :P] = rng.standard_normal((K, P)).astype(np.float32)
    b = [int(v) for v in rng.integers(1, 300, K)]
    lr = 0.1
    want, g = _oracle_weighted_sgd(theta, G[:, :P], b, lr)
    th = torch.from_numpy(theta).cuda()
    Gd = torch.from_numpy(G).cuda()
    shadow = torch.zeros(P, dtype=torch.bfloat16, device="cuda")
    omni.weighted_sgd(th, Gd, b, lr, shadow_bf16=shadow)
    torch.cuda.synchronize()
    got = th.cpu().numpy()
    assert_close(got, want, 1e-6, "theta'")
    assert_close((theta.astype(np.float64) - got) / lr, g, 1e-5, "g")
    # the bf16 copy is the fp32 result rounded to nearest even
    assert np.array_equal(shadow.float().cpu().numpy().astype(np.float64), OL.round_bf16(got))
    # without the shadow: same theta, bit for bit
    th2 = torch.from_numpy(theta).cuda()
    omni.weighted_sgd(th2, Gd, b, lr)
    torch.cuda.synchronize()
    assert torch.equal(th, th2)
    # lr = 0 leaves theta bit-identical
    th3 = torch.from_numpy(theta).cuda()
    omni.weighted_sgd(th3, Gd, b, 0.0)
    torch.cuda.synchronize()
    assert np.array_equal(th3.cpu().numpy(), theta)


def test_weighted_sgd_rejects():
    import torch
    import paper_2503_17469_amd as omni
    th = torch.zeros(128, device="cuda")
    G = torch.zeros(2, 128, device="cuda")
    for b in ([1, 0], [], list(range(1, 66))):
        with pytest.raises(omni.OmniError):
            omni.weighted_sgd(th, G, b, 0.1)
    with pytest.raises(omni.OmniError):
        omni.weighted_sgd(th, G, [1, 2], float("inf"))


@pytest.mark.parametrize("C,off", [(10, [0, 8, 32]), (100, [0, 1, 2, 700, 2048]), (1000, [0, 3, 10]), (1, [0, 5]),
                                   (65, [0, 17, 18, 40])])
def test_softmax_xent(C, off):
    import torch
    import paper_2503_17469_amd as omni
    print(f"case softmax_xent C={C} off={off}", flush=True)
    rng = np.random.default_rng(C)
    B, K = off[-1], len(off) - 1
    z = (rng.standard_normal((B, C)) * 4).astype(np.float32)
    y = rng.integers(0, C, B).astype(np.int32)
    loss_rows, dz = OL.softmax_xent(z.astype(np.float64), y)
    Lk = np.array([loss_rows[off[k]:off[k + 1]].mean() for k in range(K)])
    for k in range(K):
        dz[off[k]:off[k + 1]] /= (off[k + 1] - off[k])
    L = sum((off[k + 1] - off[k]) / B * Lk[k] for k in range(K))
    zd, yd = torch.from_numpy(z).cuda(), torch.from_numpy(y).cuda()
    dzd = torch.empty_like(zd)
    rows = torch.empty(B, device="cuda")
    lpw = torch.empty(K, device="cuda")
    loss = torch.empty(1, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    omni.softmax_xent(zd, yd, off, dzd, rows, lpw, loss, status)
    torch.cuda.synchronize()
    assert status.item() == 0
    if C > 1:
        assert_close(dzd.cpu().numpy(), dz, 1e-5, "dz")
        assert_close(rows.cpu().numpy(), loss_rows, 1e-5, "loss rows")
        assert_close(lpw.cpu().numpy(), Lk, 1e-5, "L_k")
        assert abs(loss.item() - L) <= 1e-5 * abs(L)
    else:
        assert np.abs(dzd.cpu().numpy()).max() == 0 and abs(loss.item()) == 0
    # the status word reports THIS call: a label out of range sets bit 0, and the next clean call clears it again
    if C > 1 and B > 1:
        bad = y.copy()
        bad[B // 2] = C
        omni.softmax_xent(zd, torch.from_numpy(bad).cuda(), off, dzd, rows, lpw, loss, status)
        torch.cuda.synchronize()
        assert status.item() & 1
        omni.softmax_xent(zd, yd, off, dzd, rows, lpw, loss, status)
        torch.cuda.synchronize()
        assert status.item() == 0
        assert_close(dzd.cpu().numpy(), dz, 1e-5, "dz after a call with a bad label")


@pytest.mark.parametrize("P,K,mu,wd", [(9610, 2, 0.9, 5e-4), (4206602, 4, 0.9, 5e-4), (1027, 5, 0.5, 0.0),
                                       (3, 1, 0.9, 1e-4), (113738, 16, 0.0, 5e-4)])
def test_weighted_sgd_momentum(P, K, mu, wd):
    """Four consecutive updates with the velocity carried along, against the fp64 oracle
    free-running from the same start (fp32 rounding of four steps stays far inside 1e-4)."""
    import torch
    import paper_2503_17469_amd as omni
    from oracle import optim as OO
    print(f"case weighted_sgd_momentum P={P} K={K} mu={mu} wd={wd}", flush=True)
    rng = np.random.default_rng(P * 7 + K)
    stride = (P + 63) // 64 * 64
    theta = rng.standard_normal(P).astype(np.float32)
    b = [int(v) for v in rng.integers(1, 300, K)]
    lr = 0.05
    th = torch.from_numpy(theta).cuda()
    vel = torch.zeros(P, device="cuda")
    shadow = torch.zeros(P, dtype=torch.bfloat16, device="cuda")
    ref_t, ref_v = theta.astype(np.float64), np.zeros(P)
    for s in range(4):
        G = np.zeros((K, stride), dtype=np.float32)
        G[:, :P] = rng.standard_normal((K, P)).astype(np.float32)
        omni.weighted_sgd_momentum(th, vel, torch.from_numpy(G).cuda(), b, lr, mu, wd, shadow_bf16=shadow)
        ref_t, ref_v, _ = OO.weighted_momentum_step(ref_t, ref_v, G[:, :P], b, lr, mu, wd)
    torch.cuda.synchronize()
    got_t, got_v = th.cpu().numpy(), vel.cpu().numpy()
    assert_close(got_t, ref_t, 1e-4, "theta after 4 steps")
    assert_close(got_v, ref_v, 1e-4, "velocity after 4 steps")
    assert np.array_equal(shadow.float().cpu().numpy().astype(np.float64), OL.round_bf16(got_t))


def test_weighted_sgd_momentum_degenerate_and_rejects():
    import torch
    import paper_2503_17469_amd as omni
    rng = np.random.default_rng(5)
    P, K = 1000, 3
    theta = rng.standard_normal(P).astype(np.float32)
    G = torch.from_numpy(rng.standard_normal((K, 1024)).astype(np.float32)).cuda()
    b = [3, 1, 9]
    # momentum 0, weight decay 0: the plain update, bit for bit; velocity receives the aggregate
    t1, t2 = torch.from_numpy(theta).cuda(), torch.from_numpy(theta).cuda()
    vel = torch.zeros(P, device="cuda")
    omni.weighted_sgd(t1, G, b, 0.1, P=P)
    omni.weighted_sgd_momentum(t2, vel, G, b, 0.1, 0.0, 0.0, P=P)
    torch.cuda.synchronize()
    assert torch.equal(t1, t2)
    for bad in (dict(momentum=1.0), dict(momentum=-0.1), dict(weight_decay=-1e-3), dict(momentum=float("nan"))):
        kw = dict(momentum=0.9, weight_decay=5e-4)
        kw.update(bad)
        with pytest.raises(omni.OmniError):
            omni.weighted_sgd_momentum(t2, vel, G, b, 0.1, kw["momentum"], kw["weight_decay"], P=P)
    with pytest.raises(omni.OmniError):
        omni.weighted_sgd_momentum(t2, None, G, b, 0.1, 0.9, 0.0, P=P)
