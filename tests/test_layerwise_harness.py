"""CPU check of the layer-by-layer parity harness (`tests/layerwise.py`) itself.

The harness compares what a GPU step stored with the oracle's single-layer functions.  Here the
"GPU" is a stand-in: the same networks run through an independent autograd library (torch, fp64)
with bf16 storage of every layer output, presented through the two views the harness reads
(stored outputs with folded ReLUs, gradients with respect to the value before the ReLU, a batch
norm that feeds a residual add not stored at all).  A correct pipeline must pass at the bf16
tolerance; a planted mistake in one layer's stored output, in one stored
gradient or in one worker's parameter gradient must fail at exactly that tensor.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import layers as OL

from gpu_util import fused_bn_layers
from layerwise import Layerwise
from test_oracle_step import _rand_problem, tiny_cnn, tiny_resnet
from test_oracle_store import _torch_forward_stored


class _Err(RuntimeError):
    pass


class _FakeOmni:
    OmniError = _Err

    def __init__(self, acts, grads, layers, not_stored=()):
        self.acts, self.grads, self.layers, self.not_stored = acts, grads, layers, set(not_stored)
        self.unstored = fused_bn_layers(layers)

    def _root(self, i):
        while self.layers[i]["op"] == "relu":
            i = self.layers[i]["src"]
        return i

    def _relu_of(self, r):
        for j, L in enumerate(self.layers):
            if L["op"] == "relu" and L["src"] == r:
                return j
        return None

    def net_activation(self, net, ws, layer, rows, dt):
        r = self._root(layer)
        if self.layers[r]["op"] == "bn" and r in self.unstored:
            return torch.full_like(torch.from_numpy(self.acts[r]), float("nan"))[:rows]     # never written
        j = self._relu_of(r)
        return torch.from_numpy(self.acts[r if j is None else j])[:rows]

    def net_activation_grad(self, net, ws, layer, rows, dt):
        r = self._root(layer)
        if r in self.not_stored:
            raise _Err("not stored")
        return torch.from_numpy(self.grads[r])[:rows]


class _FakeRun:
    net, ws = None, None

    def __init__(self, omni):
        self.omni = omni


def _stand_in(net, shp, cls, off, seed):
    import torch.nn.functional as F
    B = off[-1]
    theta, x, y = _rand_problem(net, shp, cls, B, seed)
    theta, x = OL.round_bf16(theta), OL.round_bf16(x)
    n = len(net)
    acts = [[] for _ in range(n)]
    grads = [[] for _ in range(n)]
    G, Lk = [], []
    for k in range(len(off) - 1):
        th = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
        xs = torch.tensor(x[off[k]:off[k + 1]], dtype=torch.float64)
        z, a = _torch_forward_stored(net, th, xs, [0, off[k + 1] - off[k]], retain=True)
        lk = F.cross_entropy(z, torch.tensor(y[off[k]:off[k + 1]], dtype=torch.long), reduction="mean")
        lk.backward()
        for li in range(n):
            acts[li].append(a[li].detach().permute(0, 2, 3, 1).reshape(a[li].shape[0], -1).numpy())
            g = a[li].grad
            g = torch.zeros_like(a[li]) if g is None else g
            gr = g.permute(0, 2, 3, 1).reshape(g.shape[0], -1).numpy()
            grads[li].append(gr if li == n - 1 else OL.round_bf16(gr))     # gradients are stored in bf16 too
        G.append(th.grad.numpy().copy())
        Lk.append(lk.item())
    acts = [np.concatenate(a).astype(np.float32) for a in acts]
    grads = [np.concatenate(g).astype(np.float32) for g in grads]
    lam = np.diff(off) / B
    got = dict(worker_grads=np.array(G), loss_per_worker=np.array(Lk), loss=float(lam @ np.array(Lk)))
    return theta, x, y, acts, grads, got


CASES = {
    "resnet": (tiny_resnet, (8, 8, 3), 5, [0, 3, 7, 12]),
    "cnn": (tiny_cnn, (8, 8, 3), 4, [0, 2, 9]),
    "mlp": (lambda: synth.mlp([24, 16, 16, 7]), (1, 1, 24), 7, [0, 3, 4, 13]),
}


@pytest.mark.parametrize("which", list(CASES))
def test_harness_accepts_a_correct_pipeline(which):
    make, shp, cls, off = CASES[which]
    net = make()
    theta, x, y, acts, grads, got = _stand_in(net, shp, cls, off, 41)
    # the CNN's first convolution is followed by a pooling: its output gradient is "not stored"
    not_stored = {0} if which == "cnn" else ()
    lw = Layerwise(_FakeRun(_FakeOmni(acts, grads, net, not_stored)), net, shp, theta, x, y, off, got, 2e-2,
                   threads=4, log=lambda *a: None)
    try:
        worst = lw.run_all()
        # the stand-in's parameter gradients come from unrounded gradients, the harness feeds the oracle the stored
        # (bf16) ones: a few-row worker's batch-norm sums differ by about a percent, everything else by less
        assert max(worst[1]) < 2e-2
        assert len(lw.worst) >= 3 * sum(1 for L in net if L["op"] in ("conv", "linear", "bn"))
    finally:
        lw.close()


@pytest.mark.parametrize("what", ["output", "gradient", "worker_grad", "bn_stat_scope"])
def test_harness_rejects_a_planted_mistake(what):
    make, shp, cls, off = CASES["resnet"]
    net = make()
    theta, x, y, acts, grads, got = _stand_in(net, shp, cls, off, 43)
    convs = [i for i, L in enumerate(net) if L["op"] == "conv"]
    target = convs[2]
    if what == "output":
        acts[target] = acts[target] * np.float32(1.05)                   # 5 % off in one layer's stored output
        expect = f"layer {target} conv output"
    elif what == "gradient":
        src = net[target]["src"]
        while net[src]["op"] == "relu":
            src = net[src]["src"]
        grads[src] = grads[src] * np.float32(0.9)                        # one tensor's stored gradient 10 % short
        expect = f"layer {src} "       # caught at that tensor: its own gradient, or the layer's parameter gradients computed from it
    elif what == "worker_grad":
        s, e = synth.param_slices(net)[target]["w"]
        got["worker_grads"][1, s:e] *= 1.04                              # one worker's gradient of one layer
        expect = f"g_1 layer {target} conv weight"
    else:
        # batch norm with the statistics of the WHOLE batch instead of each worker's own rows
        bn = next(i for i, L in enumerate(net) if L["op"] == "bn")
        X = acts[net[bn]["src"]].astype(np.float64).reshape((off[-1],) + synth.layer_shapes(net, shp)[bn])
        sl = synth.param_slices(net)[bn]
        yb = OL.bn_fwd(X, theta[sl["gamma"][0]:sl["gamma"][1]], theta[sl["beta"][0]:sl["beta"][1]])[0]
        acts[bn + 1] = OL.relu_fwd(OL.round_bf16(yb)).reshape(off[-1], -1).astype(np.float32)
        expect = f"layer {bn} bn output"
    lw = Layerwise(_FakeRun(_FakeOmni(acts, grads, net)), net, shp, theta, x, y, off, got, 2e-2, threads=4,
                   log=lambda *a: None)
    try:
        with pytest.raises(AssertionError, match=expect):
            lw.run_all()
    finally:
        lw.close()
