"""Pins for the step oracle (CPU only): finite differences, an independent autograd
library, brute-force loops, closed forms and the aggregation identity."""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import layers as L
from oracle import step as S
from oracle.controller import controller_run


def tiny_resnet():
    # conv+bn+relu, one identity block, one strided block with projection, pool, gap, fc
    return synth.resnet18(num_classes=5, widths=(4, 6), blocks=(1, 1), cin=3)


def tiny_cnn():
    return synth.cnn3(num_classes=4, hw=8, chans=(3, 4, 5, 6))


def _rand_problem(net, in_shape, classes, B, seed, bn_random=True):
    rng = np.random.default_rng(seed)
    theta = synth.he_normal_params(net, seed, bf16=False).astype(np.float64)
    # random biases / gamma / beta so every parameter's gradient is exercised
    for lay, sl in zip(net, synth.param_slices(net)):
        for name, (s, e) in sl.items():
            if name in ("b", "beta"):
                theta[s:e] = rng.standard_normal(e - s) * 0.3
            if name == "gamma":
                theta[s:e] = 1.0 + rng.standard_normal(e - s) * 0.2
    x = rng.standard_normal((B,) + tuple(in_shape))
    y = rng.integers(0, classes, size=B)
    return theta, x, y


def _objective(net, theta, x, y, off):
    """sum_k (b_k/B) * mean loss of worker k, computed only from forward passes."""
    B = off[-1]
    tot = 0.0
    for k in range(len(off) - 1):
        rows, _, _ = S.forward_backward(net, theta, x[off[k]:off[k + 1]], y[off[k]:off[k + 1]], 0.0)
        tot += (off[k + 1] - off[k]) / B * rows.mean()
    return tot


@pytest.mark.parametrize("which", ["mlp", "cnn", "resnet"])
def test_finite_differences(which):
    if which == "mlp":
        net, shp, cls, B = synth.mlp([64, 128, 10]), (1, 1, 64), 10, 32
        off = [0, 8, 32]
    elif which == "cnn":
        net, shp, cls, B = tiny_cnn(), (8, 8, 3), 4, 6
        off = [0, 2, 6]
    else:
        net, shp, cls, B = tiny_resnet(), (8, 8, 3), 5, 7
        off = [0, 3, 7]
    theta, x, y = _rand_problem(net, shp, cls, B, 5)
    res = S.sgd_step(net, theta, x, y, off, 0.1)
    rng = np.random.default_rng(0)
    idx = rng.choice(theta.size, size=min(60, theta.size), replace=False)
    # make sure every parameter tensor is sampled at least once
    for sl in synth.param_slices(net):
        for (s, e) in sl.values():
            idx = np.append(idx, rng.integers(s, e))
    h = 1e-6
    for j in idx:
        tp, tm = theta.copy(), theta.copy()
        tp[j] += h
        tm[j] -= h
        fd = (_objective(net, tp, x, y, off) - _objective(net, tm, x, y, off)) / (2 * h)
        assert abs(fd - res.grad[j]) <= 1e-6 * max(1.0, abs(fd)) + 2e-8, (which, j, fd, res.grad[j])


def _torch_forward(net, theta, x, segments):
    """The same networks written with torch's own operators (NCHW), fp64."""
    import torch.nn.functional as F
    acts = []
    pos = 0
    a_in = x.permute(0, 3, 1, 2)

    def src(i):
        return a_in if i < 0 else acts[i]

    for lay in net:
        a = src(lay["src"])
        op = lay["op"]
        if op == "linear":
            n_w = lay["cout"] * lay["cin"]
            W = theta[pos:pos + n_w].reshape(lay["cout"], lay["cin"]); pos += n_w
            b = None
            if lay["bias"]:
                b = theta[pos:pos + lay["cout"]]; pos += lay["cout"]
            flat = a.permute(0, 2, 3, 1).reshape(a.shape[0], -1)       # (h, w, c) order
            y = F.linear(flat, W, b).reshape(a.shape[0], -1, 1, 1)
        elif op == "conv":
            k = lay["k"]
            n_w = lay["cout"] * k * k * lay["cin"]
            W = theta[pos:pos + n_w].reshape(lay["cout"], k, k, lay["cin"]).permute(0, 3, 1, 2); pos += n_w
            b = None
            if lay["bias"]:
                b = theta[pos:pos + lay["cout"]]; pos += lay["cout"]
            y = F.conv2d(a, W, b, stride=lay["stride"], padding=lay["pad"])
        elif op == "relu":
            y = F.relu(a)
        elif op == "maxpool2":
            y = F.max_pool2d(a, 2, 2)
        elif op == "bn":
            c = lay["c"]
            gamma = theta[pos:pos + c]; pos += c
            beta = theta[pos:pos + c]; pos += c
            parts = [F.batch_norm(a[s0:s1], None, None, gamma, beta, training=True, eps=1e-5)
                     for s0, s1 in zip(segments[:-1], segments[1:])]
            y = torch.cat(parts, 0)
        elif op == "add":
            y = a + src(lay["src2"])
        elif op == "gap":
            y = a.mean(dim=(2, 3), keepdim=True)
        acts.append(y)
    return acts[-1].reshape(x.shape[0], -1)


@pytest.mark.parametrize("which", ["mlp", "cnn", "resnet"])
def test_against_torch_autograd(which):
    import torch.nn.functional as F
    if which == "mlp":
        net, shp, cls, B, off = synth.mlp([20, 16, 12, 7]), (1, 1, 20), 7, 11, [0, 3, 4, 11]
    elif which == "cnn":
        net, shp, cls, B, off = tiny_cnn(), (8, 8, 3), 4, 9, [0, 2, 9]
    else:
        net, shp, cls, B, off = tiny_resnet(), (8, 8, 3), 5, 10, [0, 4, 6, 10]
    theta, x, y = _rand_problem(net, shp, cls, B, 11)
    res = S.sgd_step(net, theta, x, y, off, 0.05)

    th = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    xt = torch.tensor(x, dtype=torch.float64)
    yt = torch.tensor(y, dtype=torch.long)
    z = _torch_forward(net, th, xt, off)
    # mean over ALL rows of the concatenated batch (batch norm still per segment)
    loss = F.cross_entropy(z, yt, reduction="mean")
    loss.backward()
    np.testing.assert_allclose(res.loss, loss.item(), rtol=1e-12)
    np.testing.assert_allclose(res.grad, th.grad.numpy(), rtol=1e-9, atol=1e-12)
    # per-worker mean gradients
    for k in range(len(off) - 1):
        th2 = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
        zk = _torch_forward(net, th2, xt[off[k]:off[k + 1]], [0, off[k + 1] - off[k]])
        lk = F.cross_entropy(zk, yt[off[k]:off[k + 1]], reduction="mean")
        lk.backward()
        np.testing.assert_allclose(res.loss_per_worker[k], lk.item(), rtol=1e-12)
        np.testing.assert_allclose(res.worker_grads[k], th2.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(res.params, theta - 0.05 * th.grad.numpy(), rtol=1e-12, atol=1e-14)


def test_conv_brute_force_loops():
    rng = np.random.default_rng(3)
    for (H, W, ci, co, k, s, p) in [(5, 4, 2, 3, 3, 1, 1), (6, 6, 3, 2, 3, 2, 1), (4, 4, 2, 2, 1, 2, 0)]:
        x = rng.standard_normal((2, H, W, ci))
        Wt = rng.standard_normal((co, k, k, ci))
        b = rng.standard_normal(co)
        y = L.conv_fwd(x, Wt, b, s, p)
        Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
        assert y.shape == (2, Ho, Wo, co)
        for n in range(2):
            for i in range(Ho):
                for j in range(Wo):
                    for o in range(co):
                        acc = b[o]
                        for u in range(k):
                            for v in range(k):
                                ii, jj = i * s + u - p, j * s + v - p
                                if 0 <= ii < H and 0 <= jj < W:
                                    for c in range(ci):
                                        acc += x[n, ii, jj, c] * Wt[o, u, v, c]
                        assert abs(acc - y[n, i, j, o]) < 1e-12
        # backward by brute force: dL/dx and dL/dW for L = sum(dy * y)
        dy = rng.standard_normal(y.shape)
        dx, dW, db = L.conv_bwd(x, Wt, dy, s, p)
        dx_ref = np.zeros_like(x)
        dW_ref = np.zeros_like(Wt)
        for n in range(2):
            for i in range(Ho):
                for j in range(Wo):
                    for o in range(co):
                        for u in range(k):
                            for v in range(k):
                                ii, jj = i * s + u - p, j * s + v - p
                                if 0 <= ii < H and 0 <= jj < W:
                                    for c in range(ci):
                                        dx_ref[n, ii, jj, c] += dy[n, i, j, o] * Wt[o, u, v, c]
                                        dW_ref[o, u, v, c] += dy[n, i, j, o] * x[n, ii, jj, c]
        np.testing.assert_allclose(dx, dx_ref, atol=1e-12)
        np.testing.assert_allclose(dW, dW_ref, atol=1e-12)
        np.testing.assert_allclose(db, dy.sum(axis=(0, 1, 2)), atol=1e-12)


def test_maxpool_first_max_on_ties():
    x = np.zeros((1, 2, 4, 1))
    x[0, :, :, 0] = [[1.0, 1.0, 0.0, 3.0],
                     [1.0, 0.5, 3.0, 3.0]]
    y = L.maxpool2_fwd(x)
    assert y[0, 0, :, 0].tolist() == [1.0, 3.0]
    dx = L.maxpool2_bwd(x, np.array([[[[10.0], [20.0]]]]))
    # first maximum in (dy, dx) scan order: (0,0) for the left window, (0,1) for the right one
    assert dx[0, :, :, 0].tolist() == [[10.0, 0.0, 0.0, 20.0], [0.0, 0.0, 0.0, 0.0]]


def test_softmax_xent_closed_forms():
    C = 10
    z = np.full((4, C), 3.7)
    loss, dz = L.softmax_xent(z, np.array([0, 3, 9, 5]))
    np.testing.assert_allclose(loss, math.log(C), rtol=1e-14)
    rng = np.random.default_rng(2)
    z = rng.standard_normal((50, C)) * 30            # large logits: needs the max subtraction
    y = rng.integers(0, C, 50)
    loss, dz = L.softmax_xent(z, y)
    assert np.all(np.isfinite(loss)) and np.all(loss >= 0)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-12)
    # two-class case reduces to the logistic loss
    z2 = rng.standard_normal((20, 2))
    y2 = rng.integers(0, 2, 20)
    loss2, _ = L.softmax_xent(z2, y2)
    margin = z2[np.arange(20), y2] - z2[np.arange(20), 1 - y2]
    np.testing.assert_allclose(loss2, np.log1p(np.exp(-margin)), rtol=1e-12)


def test_loss_at_init_is_about_log_classes():
    w = synth.workload(0)
    b, off = controller_run(w.T, w.B)
    res = S.sgd_step(w.layers, w.params, w.x.reshape(w.B, 1, 1, -1), w.labels, off, w.lr)
    assert 0.5 * math.log(10) < res.loss < 3 * math.log(10)


def test_batchnorm_closed_forms():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((6, 3, 3, 5)) * 3 + 2
    y, (xhat, var) = L.bn_fwd(x, np.ones(5), np.zeros(5))
    np.testing.assert_allclose(y.mean(axis=(0, 1, 2)), 0, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=(0, 1, 2)), var / (var + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(var, x.var(axis=(0, 1, 2)), rtol=1e-12)      # biased variance
    dy = rng.standard_normal(x.shape)
    dx, dgamma, dbeta = L.bn_bwd((xhat, var), rng.standard_normal(5), dy)
    np.testing.assert_allclose(dx.sum(axis=(0, 1, 2)), 0, atol=1e-10)


@pytest.mark.parametrize("which", ["mlp", "cnn", "resnet"])
def test_weighted_aggregation_equals_concatenated_batch(which):
    """sum_k (b_k/B) * (mean gradient of worker k) == mean gradient over all B rows."""
    if which == "mlp":
        net, shp, cls, B, off = synth.mlp([64, 128, 10]), (1, 1, 64), 10, 32, [0, 8, 32]
    elif which == "cnn":
        net, shp, cls, B, off = tiny_cnn(), (8, 8, 3), 4, 12, [0, 1, 5, 12]
    else:
        net, shp, cls, B, off = tiny_resnet(), (8, 8, 3), 5, 12, [0, 2, 5, 12]
    theta, x, y = _rand_problem(net, shp, cls, B, 21)
    res = S.sgd_step(net, theta, x, y, off, 0.1)
    rows, g_all, _ = S.forward_backward(net, theta, x, y, 1.0 / B, segments=off)
    scale = np.abs(g_all).max()
    assert np.abs(res.grad - g_all).max() <= 1e-12 * scale
    np.testing.assert_allclose(res.loss, rows.mean(), rtol=1e-13)
    # an UNWEIGHTED average of the worker gradients is a different vector (ragged b)
    plain = res.worker_grads.mean(axis=0)
    assert np.abs(plain - g_all).max() > 1e-6 * scale


def test_uniform_batches_reduce_to_plain_averaging():
    """b_k = B/K: lambda_k = 1/K, the step is uniform-batch synchronous SGD (equation distsgdBSP)."""
    net = synth.mlp([12, 9, 5])
    theta, x, y = _rand_problem(net, (1, 1, 12), 5, 12, 8)
    off = [0, 4, 8, 12]
    res = S.sgd_step(net, theta, x, y, off, 0.3)
    np.testing.assert_allclose(res.grad, res.worker_grads.mean(axis=0), rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(res.params, theta - 0.3 * res.worker_grads.mean(axis=0), rtol=1e-13, atol=1e-16)


def test_update_special_cases():
    net = tiny_cnn()
    theta, x, y = _rand_problem(net, (8, 8, 3), 4, 10, 13)
    off = [0, 3, 10]
    r0 = S.sgd_step(net, theta, x, y, off, 0.0)
    assert np.array_equal(r0.params, theta)                      # lr = 0 leaves theta untouched
    r1 = S.sgd_step(net, theta, x, y, [0, 10], 0.2)              # K = 1: plain mini-batch SGD
    rows, g, _ = S.forward_backward(net, theta, x, y, 1.0 / 10)
    np.testing.assert_allclose(r1.params, theta - 0.2 * g, rtol=1e-14, atol=1e-16)
    # swapping the two workers (with their rows) leaves g unchanged
    r = S.sgd_step(net, theta, x, y, off, 0.2)
    xs = np.concatenate([x[3:], x[:3]])
    ys = np.concatenate([y[3:], y[:3]])
    rs = S.sgd_step(net, theta, xs, ys, [0, 7, 10], 0.2)
    np.testing.assert_allclose(rs.grad, r.grad, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(rs.worker_grads[0], r.worker_grads[1], rtol=1e-13, atol=1e-16)


def test_round_bf16():
    v = np.array([1.0, 1.0 + 2**-8, 1.0 + 2**-7, 1.0 + 3 * 2**-8, -3.3, 0.0, 65504.0])
    r = L.round_bf16(v)
    # ties go to the even mantissa: 1+2^-8 is halfway between 1 and 1+2^-7 -> 1; 1+3*2^-8 -> 1+2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2**-7 and r[3] == 1.0 + 2**-6
    assert abs(r[4] + 3.3) <= 3.3 * 2**-8 and r[5] == 0.0
    t = torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(r, t)
    assert np.array_equal(synth.to_bf16_grid(v.astype(np.float32)).astype(np.float64), t)
