"""Seeded synthetic workloads shared by the CPU oracle's tests and the GPU path.

This package holds network *descriptions* (block lists, module splits, shapes)
and a counter-based random generator for inputs, labels and initial weights.
It contains none of the method's arithmetic (no convolution, no BN, no update
rule) and imports neither the oracle nor the HIP library.
"""
from .configs import (BLOCK_STEM, BLOCK_BASIC, BLOCK_BOTTLENECK, BLOCK_HEAD,
                      Block, ModuleSpec, Workload, get_workload, WORKLOADS,
                      block_param_shapes, module_param_count, resnet8)
from .rng import normal, uniform_int
from .init import init_module_params, minibatch, synthetic_delta

__all__ = [
    "BLOCK_STEM", "BLOCK_BASIC", "BLOCK_BOTTLENECK", "BLOCK_HEAD", "Block",
    "ModuleSpec", "Workload", "get_workload", "WORKLOADS", "block_param_shapes",
    "module_param_count", "normal", "uniform_int", "init_module_params",
    "minibatch", "synthetic_delta", "resnet8",
]
