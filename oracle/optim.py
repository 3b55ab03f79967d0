"""The optimiser the paper trains with: momentum SGD with weight decay and a stepwise
learning-rate schedule (test infrastructure).

The method's own update is plain SGD (equation bspvariableSGD); the experiments
(Section "Evaluation", list of model hyperparameters) run "SGD with momentum 0.9 and
weight decay 5e-4" with a learning rate that "decays by a factor of 10 after 15, 30 and
45 epochs" on PyTorch.  The paper prints no formula for it; the reading taken here is the
update of the framework it names:

    d  = g + weight_decay * theta          (L2 penalty folded into the gradient)
    v' = momentum * v + d                  (v starts at zero: the first step gives v' = d)
    theta' = theta - lr * v'               (no dampening, no Nesterov look-ahead)

with g the batch-size-weighted aggregate of equation bspweightedgrads.  Everything in
fp64, one statement per line of the definition.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def momentum_sgd_update(theta, velocity, grad, lr: float, momentum: float,
                        weight_decay: float) -> Tuple[np.ndarray, np.ndarray]:
    """One update from an already aggregated gradient.  Returns (theta', velocity')."""
    theta = np.asarray(theta, dtype=np.float64)
    velocity = np.asarray(velocity, dtype=np.float64)
    grad = np.asarray(grad, dtype=np.float64)
    d = grad + weight_decay * theta
    v_new = momentum * velocity + d
    theta_new = theta - lr * v_new
    return theta_new, v_new


def weighted_momentum_step(theta, velocity, worker_grads, b: Sequence[int], lr: float,
                           momentum: float, weight_decay: float):
    """Aggregate the per-worker mean gradients with lambda_k = b_k / sum_i b_i (equation
    bspweightedgrads, k ascending), then apply the momentum update.  Returns
    (theta', velocity', g)."""
    worker_grads = np.asarray(worker_grads, dtype=np.float64)
    total = float(sum(int(x) for x in b))
    g = np.zeros(worker_grads.shape[1], dtype=np.float64)
    for k in range(len(b)):
        g = g + (float(b[k]) / total) * worker_grads[k]
    theta_new, v_new = momentum_sgd_update(theta, velocity, g, lr, momentum, weight_decay)
    return theta_new, v_new, g


def lr_step_decay(lr0: float, gamma: float, milestones: Sequence[int], epoch: int) -> float:
    """Learning rate in force during `epoch` (counted from 0): lr0 times gamma once for
    every milestone already reached ("decays by a factor of 10 after 15, 30 and 45 epochs"
    = gamma 0.1, milestones (15, 30, 45))."""
    passed = sum(1 for m in milestones if epoch >= m)
    return float(lr0) * float(gamma) ** passed
