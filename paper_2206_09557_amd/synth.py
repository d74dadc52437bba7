"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only draws of weights and activations with the
distributions the workloads state (W ~ N(0, 0.02) as fp16, x ~ N(0, 1) as fp16) and the
layer shapes of the synthetic stand-ins for the OPT / LLaMA decoder layers.
"""
from __future__ import annotations

import numpy as np

# (m, n) of the four linear layers of one decoder block, per model family.
OPT_13B = {"qkv": (15360, 5120), "out": (5120, 5120), "fc1": (20480, 5120), "fc2": (5120, 20480)}
OPT_175B = {"qkv": (36864, 12288), "out": (12288, 12288), "fc1": (49152, 12288), "fc2": (12288, 49152)}
LLAMA_65B = {"qkv": (24576, 8192), "out": (8192, 8192), "gate_up": (22016, 8192), "down": (8192, 22016)}


def weights_fp16(m, n, seed, std=0.02):
    """W fp16 [m][n], iid N(0, std); drawn in fp32 in row blocks to bound host memory."""
    rng = np.random.default_rng(seed)
    W = np.empty((m, n), dtype=np.float16)
    step = max(1, (1 << 24) // n)
    for r0 in range(0, m, step):
        r1 = min(m, r0 + step)
        W[r0:r1] = (rng.standard_normal((r1 - r0, n), dtype=np.float32) * np.float32(std)).astype(np.float16)
    return W


def activations_fp16(n, seed, batch=None):
    """x fp16 [n] (or [batch][n]), iid N(0, 1)."""
    rng = np.random.default_rng(seed)
    shape = (n,) if batch is None else (batch, n)
    return rng.standard_normal(shape, dtype=np.float32).astype(np.float16)
