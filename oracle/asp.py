"""Asynchronous (parameter-server) training with variable batches, per the paper's
Algorithm 2 and equations aspweightedgrads / aspvariableSGD (test infrastructure).

Every worker k repeats: pull the model from the parameter server, compute the mean gradient
g_k of its own b_k samples at the pulled model, take a local SGD step with its own learning
rate eta_k = eta * b_k / B (the linear scaling rule of equation aspvariableSGD), push.
Workers run at different speeds, so a push may land on a server model that other workers have
changed since the pull; the number of such pushes is the staleness of the update.

On one machine the K workers are simulated: an iteration of worker k takes b_k / T_k time
units (T_k its throughput in samples per unit), pushes are processed in order of their
finishing time.  Everything below is exact (rational times) or fp64.

Readings (the paper is silent or at odds with itself):
  * order of simultaneous pushes: lower worker index first; a worker pulls again right
    after its own push, before any later push of the same instant;
  * what a push does to the server model.  Algorithm 2 prints pushToPS as REPLACING the
    server model by the worker's local model.  With workers that pull again right after
    their own push this makes every worker train a private chain (it always pulls what it
    has just pushed) and the server ends up with the chain of whoever pushed last: nothing
    is ever combined.  The background section describes workers "sending updates to update
    the globally shared model".  Default here (mode "apply"): the server adds the worker's
    local change, theta_PS <- theta_PS + (theta_local_new - theta_pulled)
    = theta_PS - eta_k * g_k(theta_pulled).  The printed form is kept as mode "overwrite";
  * evalBsz: as printed the two maps are never emptied, so once every worker has reported,
    each report re-evaluates getBsz for every worker from the latest reported times and the
    caller receives its own new size; a worker reporting before all K have reported keeps
    its size.  getBsz is the one of Algorithm 1 (dead-band relative to the new size, then
    the bounds), made integer by round-half-even; the global batch is not re-normalised
    (Algorithm 2 has no such step).
"""
from __future__ import annotations

from fractions import Fraction
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

from .step import forward_backward


def schedule(T: Sequence[int], b: Sequence[int], n_events: int) -> Tuple[List[int], List[int]]:
    """Order of the first n_events pushes and the server version each one was computed on.

    Worker k finishes its j-th iteration at time j * b_k / T_k.  Version v of the server
    model is the one after v pushes.  Returns (worker[e], pulled_version[e]); the staleness
    of push e is e - pulled_version[e].
    """
    K = len(T)
    if K < 1 or len(b) != K or any(x < 1 for x in T) or any(x < 1 for x in b) or n_events < 0:
        raise ValueError("bad schedule arguments")
    dur = [Fraction(int(b[k]), int(T[k])) for k in range(K)]
    done = [0] * K                       # iterations finished per worker
    pulled = [0] * K                     # version each worker is currently computing on
    worker, version = [], []
    for e in range(n_events):
        k = min(range(K), key=lambda j: ((done[j] + 1) * dur[j], j))
        worker.append(k)
        version.append(pulled[k])
        done[k] += 1
        pulled[k] = e + 1                # pulls right after its own push
    return worker, version


def worker_lr(lr: float, b_k: int, B: int, lr_scaling: bool = True) -> float:
    """eta_k of equation aspvariableSGD (or eta itself without the scaling rule)."""
    return lr * (b_k / B) if lr_scaling else lr


def mean_gradient(net, theta, x, labels, store=None):
    """g_k of equation aspweightedgrads and the mean loss, over the rows given."""
    n = x.shape[0]
    loss_rows, g, _ = forward_backward(net, theta, x, labels, 1.0 / n, store=store)
    return g, loss_rows.sum() / n


def run(net, theta0, batch_of: Callable[[int, int], Tuple[np.ndarray, np.ndarray]], worker: Sequence[int],
        pulled_version: Sequence[int], b: Sequence[int], B: int, lr: float, lr_scaling: bool = True,
        mode: str = "apply", store=None, grad_fn: Optional[Callable] = None):
    """Replay a push order.  batch_of(e, k) gives the (x, labels) worker k used for push e.

    Returns (versions, losses): versions[v] is the server model after v pushes,
    losses[e] the mean loss worker[e] saw at its pulled model.
    """
    if mode not in ("apply", "overwrite"):
        raise ValueError("mode")
    gf = grad_fn or (lambda th, x, y: mean_gradient(net, th, x, y, store=store))
    versions = [np.asarray(theta0, dtype=np.float64).copy()]
    losses = []
    for e, k in enumerate(worker):
        x, y = batch_of(e, k)
        if x.shape[0] != b[k]:
            raise ValueError("batch of the wrong size")
        th_pull = versions[pulled_version[e]]
        g, loss = gf(th_pull, x, y)
        eta_k = worker_lr(lr, b[k], B, lr_scaling)
        local_new = th_pull - eta_k * g
        if mode == "overwrite":
            versions.append(local_new)
        else:
            versions.append(versions[e] - eta_k * g)
        losses.append(loss)
    return versions, losses


def get_bsz(b: int, t: float, t_avg: float, deadband: float, b_min: int, b_max: int) -> int:
    """Procedure getBsz of Algorithm 1 for one worker, in doubles, one operation at a time."""
    bk = float(b)
    T = bk / t
    tau = t - t_avg
    delta = T * tau
    bs = bk - delta
    diff = bs - bk
    q = diff / bs
    if abs(q) >= deadband:
        c = min(max(bs, float(b_min)), float(b_max))
        return int(round(c))             # nearest, ties to even
    return b


class ParameterServer:
    """The batch-size bookkeeping of Algorithm 2's evalBsz (wrkB and wrkTime maps)."""

    def __init__(self, K: int, b_min: int, b_max: int, deadband: float):
        if K < 1 or b_min < 1 or b_max < b_min or not (0.0 <= deadband < 1.0):
            raise ValueError("bad arguments")
        self.K, self.b_min, self.b_max, self.deadband = K, b_min, b_max, float(deadband)
        self.wrk_b: Dict[int, int] = {}
        self.wrk_time: Dict[int, float] = {}

    def eval_bsz(self, k: int, b: int, t: float) -> int:
        if not (0 <= k < self.K) or b < 1 or not (t > 0.0) or t == float("inf"):
            raise ValueError("bad report")
        self.wrk_b[k] = b
        self.wrk_time[k] = float(t)
        if len(self.wrk_b) == self.K:
            s = 0.0
            for wid in range(self.K):
                s = s + self.wrk_time[wid]
            t_avg = s / float(self.K)
            for wid in range(self.K):
                self.wrk_b[wid] = get_bsz(self.wrk_b[wid], self.wrk_time[wid], t_avg, self.deadband,
                                          self.b_min, self.b_max)
        return self.wrk_b[k]
