"""Seeded synthetic inputs for the T-MAN hot path (weights codes, scales, zeros, activations).

This package holds only random-number plumbing and the workload shape tables.  It contains none of
the method's arithmetic (no dequantization, no table building, no packing), so both the CPU oracle's
tests and the HIP path's harness may draw their inputs from it without sharing any compute code.
"""
from .rng import splitmix64, uniform01, uniform_codes, uniform_fp16, normal_fp16, uniform_codes_torch
from .workloads import (
    LayerSpec,
    Workload,
    WORKLOADS,
    layer_tensors,
    activation,
    tensor_seed,
)

__all__ = [
    "splitmix64",
    "uniform01",
    "uniform_codes",
    "uniform_fp16",
    "normal_fp16",
    "uniform_codes_torch",
    "LayerSpec",
    "Workload",
    "WORKLOADS",
    "layer_tensors",
    "activation",
    "tensor_seed",
]
