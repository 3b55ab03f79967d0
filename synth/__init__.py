"""Seeded synthetic workloads: network shapes, parameters, batches, throughputs.

This module is shared by the CPU oracle's tests and by the GPU path's tests and
benchmark.  It holds data generation only: random tensors of the right shape and
distribution, plain descriptions of layer lists, and the rounding of generated
values onto the bf16 grid so both sides start from identical numbers.  None of
the method's arithmetic (controller, forward, backward, aggregation, update)
lives here.

The synthetic tensors stand in for the image datasets used in the paper's
evaluation (section "Implementation and Cluster Setup"); only shapes and value
distributions matter for one training step.
"""
from .nets import mlp, cnn3, resnet18, param_count, param_slices, layer_shapes, LayerList
from .data import (
    Workload,
    he_normal_params,
    make_batch,
    random_throughputs,
    throughput_walk,
    to_bf16_grid,
    workload,
    CONFIG_NAMES,
)

__all__ = [
    "mlp", "cnn3", "resnet18", "param_count", "param_slices", "layer_shapes", "LayerList",
    "Workload", "he_normal_params", "make_batch", "random_throughputs",
    "throughput_walk", "to_bf16_grid", "workload", "CONFIG_NAMES",
]
