"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times:
OPT-175B-shaped layers, q = 3, g = 128, batch 1.  The fp64 oracle computes a sample of
output rows one by one (first and last row blocks, block boundaries of the row split,
random rows); out-proj is compared on every row."""
import numpy as np
import pytest

import paper_2206_09557_amd as L
from oracle import bcq_oracle as O
from oracle import c_oracle
from paper_2206_09557_amd import synth

from gpu_util import Packed, check_parity, row_l1_bound, run

pytestmark = pytest.mark.gpu


def _sample_rows(m, rng, count=96):
    fixed = [0, 1, 15, 16, 17, m // 2 - 1, m // 2, m - 17, m - 16, m - 2, m - 1]
    # rows around the 21-way / 5-way row-block splits the launcher may choose
    for parts in (5, 21):
        for s in range(1, parts):
            rb = (m // 16) * s // parts
            fixed += [16 * rb - 1, 16 * rb, 16 * rb + 15]
    rows = np.unique(np.concatenate([np.array(fixed), rng.integers(0, m, size=count)]))
    return rows[(rows >= 0) & (rows < m)]


@pytest.mark.parametrize("name", ["fc1", "fc2", "qkv", "out"])
def test_opt175b_layer_sampled_rows(name):
    m, n = synth.OPT_175B[name]
    q, g = 3, 128
    print(f"case {name} m={m} n={n} q={q} g={g}", flush=True)
    W = synth.weights_fp16(m, n, seed=2000 + len(name) + m % 97)
    x = synth.activations_fp16(n, seed=2500 + m % 97)
    p = Packed.from_weights(W, q, g)
    del W
    print("packed", flush=True)
    y16 = run(p, x)
    y32 = run(p, x, f32_out=True)
    np.testing.assert_array_equal(y32.astype(np.float16), y16)
    rows = None if name == "out" else _sample_rows(m, np.random.default_rng(7))
    y_ref, _ = c_oracle.gemv_packed(p.bits, p.alpha, p.z, x, m, n, q, g, rows=rows)
    print("oracle done", flush=True)
    a = O.decode_alpha(p.alpha, m, n // g, q)
    bound = row_l1_bound(a, None, g)
    sel = slice(None) if rows is None else rows
    check_parity(y16[sel], y_ref, x, bound[sel])
    check_parity(y32[sel], y_ref, x, bound[sel], f32_out=True)
    # properties that hold at any size: finite everywhere, reproducible, and the mean
    # magnitude of the unsampled rows is that of the sampled ones (no dead row ranges)
    assert np.all(np.isfinite(y32))
    np.testing.assert_array_equal(run(p, x, f32_out=True), y32)
    blocks = np.abs(y32[: (m // 256) * 256]).reshape(-1, 256).mean(axis=1)
    assert blocks.min() > 0.2 * np.median(blocks)
