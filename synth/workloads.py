"""Shapes and seeded tensors of the benchmark workloads.

The layer shapes stand in for the linear layers of the LLMs the paper evaluates (Sec. 6.1 takes its
kernel shapes from the evaluated models); weights are random codes with random per-group scale and
zero, activations are standard normal.  Nothing here touches the method's arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

from . import rng

SEED_BASE = 0x2511_1248_0000_0000

# tensor kinds inside one layer
T_CODES, T_SCALES, T_ZEROS, T_ACT, T_OUTLIER = 0, 1, 2, 3, 4


@dataclass(frozen=True)
class LayerSpec:
    name: str
    M: int  # output features (rows of W)
    K: int  # input features
    act: str  # activations with the same tag are one shared tensor (Q/K/V, gate/up)


@dataclass(frozen=True)
class Workload:
    name: str
    config: int  # index into BASELINE.json "configs"
    bits: int
    group: int
    has_zero: bool
    layers: Tuple[LayerSpec, ...]
    tokens: Tuple[int, ...]  # values of N exercised
    zero_range: Tuple[float, float] = (6.0, 9.0)
    scale_range: Tuple[float, float] = (0.005, 0.02)
    outlier_frac: float = 0.0
    outlier_gain: float = 20.0
    instances: int = 1  # independent copies of the layer set (model depth, or cold-cache rotation)


_L7B = (
    LayerSpec("qkv", 12288, 4096, "attn_in"),
    LayerSpec("o", 4096, 4096, "attn_out"),
    LayerSpec("gate", 11008, 4096, "mlp_in"),
    LayerSpec("up", 11008, 4096, "mlp_in"),
    LayerSpec("down", 4096, 11008, "mlp_mid"),
)
_L3P8B = (
    LayerSpec("qkv", 9216, 3072, "attn_in"),
    LayerSpec("o", 3072, 3072, "attn_out"),
    LayerSpec("gate", 8192, 3072, "mlp_in"),
    LayerSpec("up", 8192, 3072, "mlp_in"),
    LayerSpec("down", 3072, 8192, "mlp_mid"),
)

WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in (
        Workload("tiny_w4g64", 0, 4, 64, True, (LayerSpec("lin", 256, 512, "x"),), (1,)),
        Workload("7b_w2g64", 1, 2, 64, True, _L7B, (1,), zero_range=(1.0, 2.0), instances=32),
        Workload("7b_w4g128", 2, 4, 128, True, _L7B, (1, 4, 8), outlier_frac=0.01, instances=32),
        Workload("prefill_w4g64", 3, 4, 64, True, (LayerSpec("up", 11008, 4096, "x"),), (256, 1024, 2048)),
        Workload("3p8b_w2g64", 4, 2, 64, True, _L3P8B, (1,), zero_range=(1.0, 2.0), instances=32),
        Workload("3p8b_w1g64", 4, 1, 64, False, _L3P8B, (1,), instances=32),
    )
}


def tensor_seed(w: Workload, instance: int, layer_index: int, kind: int) -> int:
    """One stream per (workload, bits, instance, layer, tensor kind)."""
    return SEED_BASE + (w.config << 40) + (w.bits << 32) + (instance << 16) + (layer_index << 4) + kind


def layer_tensors(w: Workload, instance: int, layer_index: int, device=None):
    """(codes u8 [M][K], scales fp16 [M][K/group], zeros fp16 [M][K/group] or None).

    With ``device`` set, codes are generated there with torch (same bits as the numpy definition)
    and scales/zeros are generated on the host and copied; otherwise everything is numpy.
    """
    spec = w.layers[layer_index]
    M, K, G = spec.M, spec.K, spec.K // w.group
    s = rng.uniform_fp16(tensor_seed(w, instance, layer_index, T_SCALES), M * G, *w.scale_range).reshape(M, G)
    z = None
    if w.has_zero:
        z = rng.uniform_fp16(tensor_seed(w, instance, layer_index, T_ZEROS), M * G, *w.zero_range).reshape(M, G)
    seed = tensor_seed(w, instance, layer_index, T_CODES)
    if device is None:
        q = rng.uniform_codes(seed, M * K, w.bits).reshape(M, K)
        return q, s, z
    import torch

    q = rng.uniform_codes_torch(seed, M * K, w.bits, device).reshape(M, K)
    s_t = torch.from_numpy(s).to(device)
    z_t = torch.from_numpy(z).to(device) if z is not None else None
    return q, s_t, z_t


def activation(w: Workload, instance: int, layer_index: int, N: int) -> np.ndarray:
    """fp16 [N][K] ~ N(0,1); layers with the same activation tag get the same tensor.  With
    ``outlier_frac`` > 0, ceil(frac*K) seeded channels (the same for every token) are multiplied by
    ``outlier_gain`` before the rounding to fp16."""
    spec = w.layers[layer_index]
    first = next(i for i, l in enumerate(w.layers) if l.act == spec.act)
    K = spec.K
    gain = np.ones(K, dtype=np.float64)
    if w.outlier_frac > 0.0:
        n_out = int(np.ceil(w.outlier_frac * K))
        keys = rng.splitmix64(tensor_seed(w, instance, first, T_OUTLIER), 0, K)
        gain[np.argsort(keys, kind="stable")[:n_out]] = w.outlier_gain
    x = rng.normal_fp16(tensor_seed(w, instance, first, T_ACT), N * K, np.tile(gain, N))
    return x.reshape(N, K)
