"""Seeded tensors and throughput traces for the benchmark workloads (no method arithmetic)."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

from . import nets

CONFIG_NAMES = ("tiny_mlp", "mlp3072", "cnn3", "resnet18", "cnn3_dynamic")


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Return fp32 values moved to the nearest bf16-representable number (ties to even).

    Used only so that generated inputs and initial weights are exactly
    representable in bf16 and both the oracle and the GPU path start from
    bit-identical values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def he_normal_params(layers, seed: int, bf16: bool) -> np.ndarray:
    """Flat fp32 parameter vector: weights N(0, 2/fan_in), biases 0, gamma 1, beta 0."""
    rng = np.random.default_rng(seed)
    P = nets.param_count(layers)
    theta = np.zeros(P, dtype=np.float32)
    for L, sl in zip(layers, nets.param_slices(layers)):
        if L["op"] == "linear":
            fan_in = L["cin"]
        elif L["op"] == "conv":
            fan_in = L["cin"] * L["k"] * L["k"]
        elif L["op"] == "bn":
            s, e = sl["gamma"]
            theta[s:e] = 1.0
            continue
        else:
            continue
        s, e = sl["w"]
        w = rng.standard_normal(e - s).astype(np.float32) * np.float32(np.sqrt(2.0 / fan_in))
        theta[s:e] = to_bf16_grid(w) if bf16 else w
    return theta


def make_batch(seed: int, B: int, in_shape: Tuple[int, int, int], classes: int, bf16: bool):
    """x ~ N(0,1) of shape [B, H, W, C] (fp32, on the bf16 grid if asked), labels uniform."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B,) + tuple(in_shape)).astype(np.float32)
    if bf16:
        x = to_bf16_grid(x)
    y = rng.integers(0, classes, size=B, dtype=np.int32)
    return x, y


def random_throughputs(seed: int, K: int, force_spread: bool = False) -> List[int]:
    """Integer throughputs in milli-units, uniform in [1000, 8000] (an up-to-8x spread)."""
    rng = np.random.default_rng(seed)
    T = rng.integers(1000, 8001, size=K)
    if force_spread and K >= 2:
        T[int(np.argmin(T))] = 1000
        T[int(np.argmax(T))] = 8000
    return [int(t) for t in T]


def throughput_walk(seed: int, K: int, steps: int) -> List[List[int]]:
    """Per-step throughputs: a bounded integer random walk inside [1000, 8000]."""
    rng = np.random.default_rng(seed)
    T = rng.integers(1000, 8001, size=K)
    out = [[int(t) for t in T]]
    for _ in range(steps - 1):
        T = np.clip(T + rng.integers(-250, 251, size=K), 1000, 8000)
        out.append([int(t) for t in T])
    return out


@dataclass
class Workload:
    name: str
    layers: list
    in_shape: Tuple[int, int, int]
    classes: int
    dtype: str            # "f32" or "bf16" (bf16 operands, fp32 accumulate, fp32 master params)
    K: int
    B: int
    T: List[int]
    lr: float
    seed: int
    params: np.ndarray = field(repr=False, default=None)
    x: np.ndarray = field(repr=False, default=None)
    labels: np.ndarray = field(repr=False, default=None)

    @property
    def P(self) -> int:
        return nets.param_count(self.layers)


def workload(index: int, B: int | None = None, K: int | None = None, with_data: bool = True) -> Workload:
    """The five benchmark configurations; seed = 1000 + index.  B / K may be
    overridden to get a smaller instance of the same shape family."""
    seed = 1000 + index
    if index == 0:
        layers, shp, cls, dt = nets.mlp([64, 128, 10]), (1, 1, 64), 10, "f32"
        K0, B0, T = 2, 32, [1000, 3000]
    elif index == 1:
        layers, shp, cls, dt = nets.mlp([3072, 1024, 1024, 10]), (1, 1, 3072), 10, "f32"
        K0, B0, T = 4, 480, [1000, 2000, 4000, 8000]
    elif index == 2:
        layers, shp, cls, dt = nets.cnn3(10), (32, 32, 3), 10, "bf16"
        K0, B0, T = 8, 1024, None
    elif index == 3:
        layers, shp, cls, dt = nets.resnet18(100), (32, 32, 3), 100, "bf16"
        K0, B0, T = 8, 2048, None
    elif index == 4:
        layers, shp, cls, dt = nets.cnn3(10), (32, 32, 3), 10, "bf16"
        K0, B0, T = 16, 2048, None
    else:
        raise ValueError(index)
    K = K0 if K is None else K
    B = B0 if B is None else B
    if T is None or K != K0:
        T = random_throughputs(seed, K, force_spread=(index == 3))
    w = Workload(CONFIG_NAMES[index], layers, shp, cls, dt, K, B, T, 0.1, seed)
    if with_data:
        w.params = he_normal_params(layers, seed + 17, dt == "bf16")
        w.x, w.labels = make_batch(seed + 31, B, shp, cls, dt == "bf16")
    return w
