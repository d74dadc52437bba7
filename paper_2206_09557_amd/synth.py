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


def weights_fp16(m, n, seed, std=0.02, workers=8):
    """W fp16 [m][n], iid N(0, std).  Row blocks of a fixed size are drawn in fp32 from
    child streams of `seed`, so the matrix does not depend on the number of workers."""
    W = np.empty((m, n), dtype=np.float16)
    step = max(1, (1 << 22) // n)
    starts = list(range(0, m, step))
    children = np.random.SeedSequence(seed).spawn(len(starts))

    def fill(idx):
        r0 = starts[idx]
        r1 = min(m, r0 + step)
        rng = np.random.default_rng(children[idx])
        W[r0:r1] = (rng.standard_normal((r1 - r0, n), dtype=np.float32) * np.float32(std)).astype(np.float16)

    if len(starts) == 1 or workers <= 1:
        for i in range(len(starts)):
            fill(i)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(fill, range(len(starts))))
    return W


def activations_fp16(n, seed, batch=None):
    """x fp16 [n] (or [batch][n]), iid N(0, 1)."""
    rng = np.random.default_rng(seed)
    shape = (n,) if batch is None else (batch, n)
    return rng.standard_normal(shape, dtype=np.float32).astype(np.float16)
