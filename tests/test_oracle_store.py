"""Pins for the step oracle's bf16 storage model (`store=round_bf16`), CPU only.

Every bf16 parity verdict is graded against `sgd_step(..., store=round_bf16)`: each layer output
except the logits is rounded to bf16 as it is stored, the layers after it read the stored values,
the backward pass takes its ReLU masks, pooling arg-maxima and batch-norm inputs from the stored
values, and rounding itself has derivative one.  Pinned here by

  * the same networks written with an independent autograd library (torch, fp64) with a
    straight-through rounding y + (bf16(y) - y).detach() after every layer but the last;
  * hand-worked cases in which the rounding changes a discrete decision (a pooling arg-maximum, a
    ReLU mask), where the stored-value model and exact arithmetic give different gradients;
  * the logits exception: the last layer's output is NOT rounded.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import layers as L
from oracle import step as S

from test_oracle_step import _rand_problem, _torch_forward, tiny_cnn, tiny_resnet


def _torch_bf16(y):
    # fp64 -> fp32 -> bf16 (nearest even) -> fp64: a bf16 store of an fp32 result
    return y.detach().to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _torch_forward_stored(net, theta, x, segments, retain=False):
    """_torch_forward with every layer output but the last replaced, as it is produced, by its
    bf16 rounding (straight-through: the rounding passes gradients unchanged)."""
    import torch.nn.functional as F
    acts = []
    pos = 0
    a_in = x.permute(0, 3, 1, 2)

    def src(i):
        return a_in if i < 0 else acts[i]

    for li, lay in enumerate(net):
        a = src(lay["src"])
        op = lay["op"]
        if op == "linear":
            n_w = lay["cout"] * lay["cin"]
            W = theta[pos:pos + n_w].reshape(lay["cout"], lay["cin"]); pos += n_w
            b = None
            if lay["bias"]:
                b = theta[pos:pos + lay["cout"]]; pos += lay["cout"]
            flat = a.permute(0, 2, 3, 1).reshape(a.shape[0], -1)
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
        if li != len(net) - 1:
            y = y + (_torch_bf16(y) - y).detach()
        if retain:
            y.retain_grad()
        acts.append(y)
    return acts[-1].reshape(x.shape[0], -1), acts


@pytest.mark.parametrize("which", ["mlp", "cnn", "resnet"])
def test_store_model_against_straight_through_autograd(which):
    import torch.nn.functional as F
    if which == "mlp":
        net, shp, cls, B, off = synth.mlp([24, 16, 16, 7]), (1, 1, 24), 7, 13, [0, 3, 4, 13]
    elif which == "cnn":
        net, shp, cls, B, off = tiny_cnn(), (8, 8, 3), 4, 9, [0, 2, 9]
    else:
        net, shp, cls, B, off = tiny_resnet(), (8, 8, 3), 5, 10, [0, 4, 6, 10]
    theta, x, y = _rand_problem(net, shp, cls, B, 31)
    # start on the bf16 grid as the parity tests do
    theta = L.round_bf16(theta)
    x = L.round_bf16(x)
    res = S.sgd_step(net, theta, x, y, off, 0.05, store=L.round_bf16, keep_acts=True)
    exact = S.sgd_step(net, theta, x, y, off, 0.05)
    xt = torch.tensor(x, dtype=torch.float64)
    yt = torch.tensor(y, dtype=torch.long)
    K = len(off) - 1
    g_sum = np.zeros_like(theta)
    for k in range(K):
        th = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
        zk, acts = _torch_forward_stored(net, th, xt[off[k]:off[k + 1]], [0, off[k + 1] - off[k]])
        lk = F.cross_entropy(zk, yt[off[k]:off[k + 1]], reduction="mean")
        lk.backward()
        # every stored activation is the same bf16 value on both sides (rounding decisions included)
        for li in range(len(net)):
            a = acts[li].detach().permute(0, 2, 3, 1).numpy()
            np.testing.assert_array_equal(a, res.acts[k][li].reshape(a.shape) if li != len(net) - 1 else a)
            if li != len(net) - 1:
                assert np.array_equal(a, L.round_bf16(a)), "stored values lie on the bf16 grid"
        np.testing.assert_allclose(res.acts[k][-1].reshape(zk.shape), zk.detach().numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(res.loss_per_worker[k], lk.item(), rtol=1e-12)
        np.testing.assert_allclose(res.worker_grads[k], th.grad.numpy(), rtol=1e-9, atol=1e-12)
        g_sum += (off[k + 1] - off[k]) / B * th.grad.numpy()
    np.testing.assert_allclose(res.grad, g_sum, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(res.params, theta - 0.05 * g_sum, rtol=1e-12, atol=1e-14)
    # the storage model is not a no-op: it moves the gradient by about bf16's resolution, and by no more
    d = np.linalg.norm(res.grad - exact.grad) / np.linalg.norm(exact.grad)
    assert 1e-5 < d < 0.2, d


def test_logits_are_not_rounded_but_hidden_outputs_are():
    net = synth.mlp([4, 3, 2])          # linear, relu, linear
    theta = np.zeros(synth.param_count(net))
    sl = synth.param_slices(net)
    W0 = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 0, 1.0, 0]])
    W1 = np.array([[1.0, 1.0, 1.0], [0.5, 0.0, 0.0]])
    theta[sl[0]["w"][0]:sl[0]["w"][1]] = W0.ravel()
    theta[sl[2]["w"][0]:sl[2]["w"][1]] = W1.ravel()
    # 1 + 2^-10 is not a bf16 value (8 significant bits): stored as 1; 2^-10 alone is one
    x = np.array([[1.0 + 2.0 ** -10, 2.0 ** -10, 1.0, 0.0]]).reshape(1, 1, 1, 4)
    _, _, acts = S.forward_backward(net, theta, x, np.array([0]), 1.0, store=L.round_bf16, keep_acts=True)
    assert acts[0].ravel().tolist() == [1.0, 2.0 ** -10, 1.0]              # hidden output rounded as stored
    assert acts[1].ravel().tolist() == [1.0, 2.0 ** -10, 1.0]
    # logits computed from the STORED hidden values and kept unrounded: 2 + 2^-10 has 12 significant bits
    assert acts[2].ravel().tolist() == [2.0 + 2.0 ** -10, 0.5]
    _, _, acts_exact = S.forward_backward(net, theta, x, np.array([0]), 1.0, keep_acts=True)
    assert acts_exact[2].ravel().tolist() == [2.0 + 2.0 ** -9, 0.5 + 2.0 ** -11]


def test_rounding_moves_a_pooling_argmax():
    """Window (1, 1 + 2^-9, 0, 0): exact arithmetic sends the gradient to the second entry; both
    entries are stored as 1 in bf16, so the stored-value model sends it to the FIRST maximum."""
    net = [dict(op="conv", src=-1, cin=1, cout=1, k=1, stride=1, pad=0, bias=False),
           dict(op="maxpool2", src=0),
           dict(op="linear", src=1, cin=1, cout=2, bias=False)]
    theta = np.array([1.0, 1.0, -1.0])          # conv weight 1; logits (p, -p)
    x = np.zeros((1, 2, 2, 1))
    x[0, 0, 0, 0], x[0, 0, 1, 0] = 1.0, 1.0 + 2.0 ** -9
    y = np.array([1])
    # dL/dp = softmax_0 * 1 + (softmax_1 - 1) * (-1) = 2 * softmax_0 (two logits p and -p, label 1)
    for store, p, winner in ((None, 1.0 + 2.0 ** -9, (0, 1)), (L.round_bf16, 1.0, (0, 0))):
        _, g, acts = S.forward_backward(net, theta, x, y, 1.0, store=store, keep_acts=True)
        assert acts[1].ravel().tolist() == [p]
        dp = 2.0 / (1.0 + np.exp(-2.0 * p))
        # the conv weight's gradient = dL/dp * (the input value at the window entry that won)
        assert g[0] == pytest.approx(dp * x[0, winner[0], winner[1], 0], rel=1e-12)
    # and the two differ by the factor 1 + 2^-9 (beyond the small change of dp), visibly
    _, g_exact, _ = S.forward_backward(net, theta, x, y, 1.0)
    _, g_store, _ = S.forward_backward(net, theta, x, y, 1.0, store=L.round_bf16)
    assert g_exact[0] != g_store[0]


def test_rounding_moves_a_relu_mask():
    """A pre-activation of 2^-140 is positive in fp64 and stored as 0 in bf16 (below half of the
    smallest subnormal, 2^-134): the stored-value model's ReLU derivative there is 0."""
    net = synth.mlp([1, 1, 2])
    net[0]["bias"] = False
    net[2]["bias"] = False
    theta = np.array([2.0 ** -140, 1.0, -1.0])
    x = np.ones((1, 1, 1, 1))
    y = np.array([0])
    _, g_exact, _ = S.forward_backward(net, theta, x, y, 1.0)
    _, g_store, acts = S.forward_backward(net, theta, x, y, 1.0, store=L.round_bf16, keep_acts=True)
    assert acts[0].ravel().tolist() == [0.0]
    # logits (h, -h) with h ~ 0: softmax = (1/2, 1/2); dL/dh = (1/2 - 1) - (1/2) = -1; dh/dw0 = x = 1 where the mask is open
    assert g_exact[0] == pytest.approx(-1.0, abs=1e-12)
    assert g_store[0] == 0.0
    # the second layer's own gradient is h * (softmax - onehot): 0 either way up to 2^-140
    assert abs(g_exact[1]) < 1e-40 and g_store[1] == 0.0
