"""One synchronous dynamic-batching SGD step, per the paper's Algorithm 1 (test infrastructure).

For every worker k separately: forward and backward on its own rows of the
concatenated batch, giving the mean loss L_k and mean gradient g_k over its
b_k samples (the gradient line of procedure Train).  Then the weighted
aggregation of equation bspweightedgrads, g = sum_k lambda_k g_k with
lambda_k = b_k / sum_i b_i, and the update of equation bspvariableSGD,
theta <- theta - eta * g.  Everything in fp64.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np

from . import layers as L


def _param_views(net, theta):
    """Per layer dict name -> array view into the flat parameter vector."""
    out = []
    pos = 0
    for lay in net:
        d = {}
        op = lay["op"]
        if op == "linear":
            n = lay["cout"] * lay["cin"]
            d["w"] = (pos, (lay["cout"], lay["cin"])); pos += n
            if lay["bias"]:
                d["b"] = (pos, (lay["cout"],)); pos += lay["cout"]
        elif op == "conv":
            shp = (lay["cout"], lay["k"], lay["k"], lay["cin"])
            d["w"] = (pos, shp); pos += int(np.prod(shp))
            if lay["bias"]:
                d["b"] = (pos, (lay["cout"],)); pos += lay["cout"]
        elif op == "bn":
            d["gamma"] = (pos, (lay["c"],)); pos += lay["c"]
            d["beta"] = (pos, (lay["c"],)); pos += lay["c"]
        out.append(d)
    assert pos == theta.size, (pos, theta.size)
    return out


def _get(theta, spec):
    pos, shp = spec
    return theta[pos:pos + int(np.prod(shp))].reshape(shp)


def _put(g, spec, val):
    pos, shp = spec
    g[pos:pos + int(np.prod(shp))] += np.asarray(val, dtype=np.float64).reshape(-1)


def forward_backward(net, theta, x, labels, loss_scale, segments=None, store: Optional[Callable] = None,
                     keep_acts: bool = False):
    """Forward and backward over the rows given.

    The scalar objective is loss_scale * sum_rows loss_row, so loss_scale = 1/n
    yields the mean loss and mean gradient over these n rows.  `segments`
    (prefix offsets within x) makes batch norm use each segment's own
    statistics; None means all rows form one segment.  `store`, if given, is
    applied to every layer output except the logits as it is written (model of
    a pipeline that stores activations in bf16 and keeps the logits in fp32), so
    that ReLU masks and pooling arg-maxima are decided on the stored values.

    Returns (per-row losses, gradient [P], activations list or None)."""
    theta = np.asarray(theta, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    if segments is None:
        segments = [0, n]
    views = _param_views(net, theta)
    st = store if store is not None else (lambda a: a)

    acts: List[np.ndarray] = []
    caches: List = []

    def src(i):
        return x if i < 0 else acts[i]

    for lay, pv in zip(net, views):
        a = src(lay["src"])
        op = lay["op"]
        cache = None
        if op == "linear":
            a2 = a.reshape(n, -1)
            y = L.linear_fwd(a2, _get(theta, pv["w"]), _get(theta, pv["b"]) if "b" in pv else None)
            y = y.reshape(n, 1, 1, -1)
        elif op == "conv":
            y = L.conv_fwd(a, _get(theta, pv["w"]), _get(theta, pv["b"]) if "b" in pv else None,
                           lay["stride"], lay["pad"])
        elif op == "relu":
            y = L.relu_fwd(a)
        elif op == "maxpool2":
            y = L.maxpool2_fwd(a)
        elif op == "bn":
            y = np.empty_like(a)
            cache = []
            for s0, s1 in zip(segments[:-1], segments[1:]):
                ys, c = L.bn_fwd(a[s0:s1], _get(theta, pv["gamma"]), _get(theta, pv["beta"]))
                y[s0:s1] = ys
                cache.append(c)
        elif op == "add":
            y = a + src(lay["src2"])
        elif op == "gap":
            y = L.gap_fwd(a)
        else:
            raise ValueError(op)
        acts.append(st(y) if lay is not net[-1] else y)
        caches.append(cache)

    z = acts[-1].reshape(n, -1)
    loss_rows, dz = L.softmax_xent(z, np.asarray(labels))
    dz = dz * loss_scale

    g = np.zeros(theta.size, dtype=np.float64)
    dacts: List[Optional[np.ndarray]] = [None] * len(net)
    dacts[-1] = dz.reshape(acts[-1].shape)

    def give(i, d):
        if i < 0:
            return
        dacts[i] = d if dacts[i] is None else dacts[i] + d

    for li in range(len(net) - 1, -1, -1):
        lay, pv = net[li], views[li]
        dy = dacts[li]
        if dy is None:
            continue
        a = src(lay["src"])
        op = lay["op"]
        if op == "linear":
            a2 = a.reshape(n, -1)
            dx, dW, db = L.linear_bwd(a2, _get(theta, pv["w"]), dy.reshape(n, -1))
            _put(g, pv["w"], dW)
            if "b" in pv:
                _put(g, pv["b"], db)
            give(lay["src"], dx.reshape(a.shape))
        elif op == "conv":
            dx, dW, db = L.conv_bwd(a, _get(theta, pv["w"]), dy, lay["stride"], lay["pad"])
            _put(g, pv["w"], dW)
            if "b" in pv:
                _put(g, pv["b"], db)
            give(lay["src"], dx)
        elif op == "relu":
            give(lay["src"], L.relu_bwd(a, dy))
        elif op == "maxpool2":
            give(lay["src"], L.maxpool2_bwd(a, dy))
        elif op == "bn":
            dx = np.empty_like(a)
            gamma = _get(theta, pv["gamma"])
            for (s0, s1), c in zip(zip(segments[:-1], segments[1:]), caches[li]):
                dxs, dgam, dbet = L.bn_bwd(c, gamma, dy[s0:s1])
                dx[s0:s1] = dxs
                _put(g, pv["gamma"], dgam)
                _put(g, pv["beta"], dbet)
            give(lay["src"], dx)
        elif op == "add":
            give(lay["src"], dy)
            give(lay["src2"], dy)
        elif op == "gap":
            give(lay["src"], L.gap_bwd(a, dy))
    return loss_rows, g, (acts if keep_acts else None)


@dataclass
class StepResult:
    loss_per_worker: np.ndarray        # L_k, mean loss of worker k
    loss: float                        # sum_k lambda_k L_k
    worker_grads: np.ndarray           # g_k, [K, P], mean gradient of worker k
    grad: np.ndarray                   # g = sum_k lambda_k g_k
    params: np.ndarray                 # theta - lr * g
    acts: Optional[list] = field(default=None, repr=False)   # per worker, per layer


def sgd_step(net, theta, x, labels, off: Sequence[int], lr: float, store=None, keep_acts=False,
             pmap=map) -> StepResult:
    """One weighted-aggregation SGD step over K workers whose rows are
    x[off[k]:off[k+1]].  The workers' passes are independent of each other; `pmap` (default: the
    builtin map, one worker after the other) lets a caller run them side by side, e.g. a thread
    pool's map.  The aggregation below is the same either way."""
    theta = np.asarray(theta, dtype=np.float64)
    K = len(off) - 1
    B = off[K] - off[0]
    Lk = np.zeros(K)
    gk = np.zeros((K, theta.size))
    acts = []

    def worker(k):
        s0, s1 = off[k], off[k + 1]
        return forward_backward(net, theta, x[s0:s1], labels[s0:s1], 1.0 / (s1 - s0), store=store,
                                keep_acts=keep_acts)

    for k, (loss_rows, g, a) in enumerate(pmap(worker, range(K))):
        Lk[k] = loss_rows.sum() / (off[k + 1] - off[k])
        gk[k] = g
        acts.append(a)
    g = np.zeros(theta.size)
    loss = 0.0
    for k in range(K):
        lam = (off[k + 1] - off[k]) / B
        g += lam * gk[k]
        loss += lam * Lk[k]
    return StepResult(Lk, loss, gk, g, theta - lr * g, acts if keep_acts else None)
