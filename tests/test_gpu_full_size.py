"""GPU parity at the full workload sizes, in the launch configuration bench.py times:
OPT-175B-shaped layers (q = 3, g = 128; every row of every layer, and the small-batch
sweep 2..32 on FC1 through the lookup path), OPT-13B-shaped layers (q = 4, g = 128) and
LLaMA-65B-shaped layers with per-group offsets over a (q, g) sweep, batch 1.  Where rows are
sampled, the fp64 oracle computes them one by one (first and last row blocks, block
boundaries of the row splits, random rows)."""
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
def test_opt175b_layer_all_rows(name):
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
    rows = None   # every row: the oracle takes about a second per layer on the machine's cores
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


def _check_layer(m, n, q, g, mode, seed, all_rows=False):
    W = synth.weights_fp16(m, n, seed=seed)
    x = synth.activations_fp16(n, seed=seed + 500)
    p = Packed.from_weights(W, q, g, mode)
    del W
    y16 = run(p, x)
    y32 = run(p, x, f32_out=True)
    np.testing.assert_array_equal(y32.astype(np.float16), y16)
    rows = None if all_rows else _sample_rows(m, np.random.default_rng(seed))
    y_ref, _ = c_oracle.gemv_packed(p.bits, p.alpha, p.z, x, m, n, q, g, rows=rows)
    gc = n if g == 0 else g
    a = O.decode_alpha(p.alpha, m, n // gc, q)
    z = None if p.z is None else O.decode_z(p.z, m, n // gc)
    bound = row_l1_bound(a, z, gc)
    sel = slice(None) if rows is None else rows
    check_parity(y16[sel], y_ref, x, bound[sel])
    check_parity(y32[sel], y_ref, x, bound[sel], f32_out=True)
    assert np.all(np.isfinite(y32))
    np.testing.assert_array_equal(run(p, x, f32_out=True), y32)


@pytest.mark.parametrize("name", ["qkv", "out", "fc1", "fc2"])
def test_opt13b_layer_sampled_rows(name):
    m, n = synth.OPT_13B[name]
    print(f"case opt13b {name} m={m} n={n} q=4 g=128", flush=True)
    _check_layer(m, n, 4, 128, L.LUTGEMM_Q_GREEDY, seed=1000 + len(name) + m % 89)


# (layer, q, g): the sweep q in {2,3,4} x g in {32,64,128,row-wise}, spread over the four
# LLaMA-65B layer shapes; gate_up / down have n or m = 22016 = 21.5 tiles of 1024 columns.
LLAMA_CASES = [("qkv", 3, 128), ("qkv", 2, 32), ("out", 4, 64), ("out", 2, 0), ("gate_up", 4, 128), ("gate_up", 3, 32),
               ("gate_up", 2, 64), ("down", 3, 0), ("down", 4, 32), ("down", 3, 64), ("down", 2, 128), ("qkv", 4, 0)]


@pytest.mark.parametrize("name,q,g", LLAMA_CASES)
def test_llama65b_layer_with_offset_sampled_rows(name, q, g):
    m, n = synth.LLAMA_65B[name]
    print(f"case llama65b {name} m={m} n={n} q={q} g={g} uniform->BCQ with offset", flush=True)
    _check_layer(m, n, q, g, L.LUTGEMM_Q_UNIFORM_RTN, seed=4000 + 7 * q + g + m % 83)


_FC1 = {}


def _fc1_packed():
    """The FC1-shaped layer of the batch sweep, packed once for all its cases."""
    if not _FC1:
        m, n = synth.OPT_175B["fc1"]
        W = synth.weights_fp16(m, n, seed=5000)
        p = Packed.from_weights(W, 3, 128)
        del W
        a = O.decode_alpha(p.alpha, m, n // 128, 3)
        _FC1["p"], _FC1["bound"] = p, row_l1_bound(a, None, 128)
    return _FC1["p"], _FC1["bound"]


@pytest.mark.parametrize("batch", [2, 3, 4, 8, 16, 32])
def test_small_batch_sweep_on_fc1_shape_lookup_path(batch):
    # the small-batch sweep of the workload list (paper section 6) through the lookup path
    # alone (no LUTGEMM_PATH_AUTO), in the grids bench.py times: every vector, every row
    m, n = synth.OPT_175B["fc1"]
    q, g = 3, 128
    p, bound = _fc1_packed()
    grids = {w: L.lutgemm_plan_grid(m, n, q, g, w) for w in (1, 2, 4)}
    print(f"case batch fc1 m={m} n={n} batch={batch} grids={grids}", flush=True)
    X = synth.activations_fp16(n, seed=5500 + batch, batch=batch)
    Y = run(p, X, f32_out=True)
    Y16 = run(p, X)
    np.testing.assert_array_equal(Y.astype(np.float16), Y16)
    Yref, _ = c_oracle.gemv_packed(p.bits, p.alpha, None, X, m, n, q, g)
    print("oracle done", flush=True)
    for b in range(batch):
        check_parity(Y[b], Yref[b], X[b], bound, f32_out=True)
        check_parity(Y16[b], Yref[b], X[b], bound)


@pytest.mark.parametrize("batch", [4, 32])
def test_mfma_path_on_fc1_shape(batch):
    # config 5 through the matrix-core path, in the launch configuration bench.py times
    m, n = synth.OPT_175B["fc1"]
    q, g = 3, 128
    print(f"case mfma fc1 m={m} n={n} batch={batch}", flush=True)
    p, bound = _fc1_packed()
    X = synth.activations_fp16(n, seed=5600 + batch, batch=batch)
    Y = run(p, X, f32_out=True, mfma=True)
    Yref, _ = c_oracle.gemv_packed(p.bits, p.alpha, None, X, m, n, q, g)
    for b in range(batch):
        check_parity(Y[b], Yref[b], X[b], bound, f32_out=True)


@pytest.mark.parametrize("batch", [1, 8])
def test_dequant_mfma_kernel_on_fc1_shape(batch):
    # the comparison kernel of the small-batch workload at the size it is timed on, every row
    m, n = synth.OPT_175B["fc1"]
    q, g = 3, 128
    print(f"case dequant fc1 m={m} n={n} batch={batch}", flush=True)
    p, bound = _fc1_packed()
    X = synth.activations_fp16(n, seed=5800 + batch, batch=batch)
    Y = run(p, X, f32_out=True, dequant=True)
    Yref, _ = c_oracle.gemv_packed(p.bits, p.alpha, None, X, m, n, q, g)
    for b in range(batch):
        check_parity(Y[b], Yref[b], X[b], bound, f32_out=True, fp16_weights=True)


def test_mfma_path_llama65b_down_with_offset():
    m, n = synth.LLAMA_65B["down"]
    q, g = 4, 128
    print(f"case mfma llama down m={m} n={n}", flush=True)
    W = synth.weights_fp16(m, n, seed=5700)
    p = Packed.from_weights(W, q, g, L.LUTGEMM_Q_UNIFORM_RTN)
    del W
    X = synth.activations_fp16(n, seed=5701, batch=8)
    Y = run(p, X, f32_out=True, mfma=True)
    rows = _sample_rows(m, np.random.default_rng(7))
    a = O.decode_alpha(p.alpha, m, n // g, q)
    z = O.decode_z(p.z, m, n // g)
    bound = row_l1_bound(a, z, g)
    Yref, _ = c_oracle.gemv_packed(p.bits, p.alpha, p.z, X, m, n, q, g, rows=rows)
    for b in range(8):
        check_parity(Y[b][rows], Yref[b], X[b], bound[rows], f32_out=True)
