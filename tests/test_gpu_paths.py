"""GPU parity for the kernel paths that only long rows reach: K groups of several tiles
(a workgroup walks more than one table set and carries row sums from tile to tile) in the
GEMV, pair and quad kernels, crossed with offsets, more than four planes, every scale
mode and the shared-scale layout; and row ranges longer than the running sums in LDS cover
(pair and quad kernels).  Every case first asks the library which grid it plans
(lutgemm_plan_grid) and asserts that the path meant is the path reached; all rows are then
compared with the fp64 C oracle."""
import numpy as np
import pytest

import paper_2206_09557_amd as L
from oracle import bcq_oracle as O
from oracle import c_oracle
from paper_2206_09557_amd import synth

from gpu_util import Packed, check_parity, row_l1_bound, run

pytestmark = pytest.mark.gpu

MODES = {"greedy": L.LUTGEMM_Q_GREEDY, "greedy_z": L.LUTGEMM_Q_GREEDY_MEAN_OFFSET, "rtn": L.LUTGEMM_Q_UNIFORM_RTN}


def _bounds(p):
    g = p.n if p.g == 0 else p.g
    a = O.decode_alpha(p.alpha, p.m, p.n // g, p.q)
    z = None if p.z is None else O.decode_z(p.z, p.m, p.n // g)
    return row_l1_bound(a, z, g)


def _check_all_rows(p, x, shared=False):
    """fp32 and fp16 outputs of the lookup path against the C oracle on every row."""
    xs = x if x.ndim == 2 else x[None, :]
    y_ref, _ = c_oracle.gemv_packed(p.bits, p.alpha, p.z, xs, p.m, p.n, p.q, p.g)
    bound = _bounds(p)
    y32 = run(p, x, f32_out=True, shared=shared)
    y16 = run(p, x, shared=shared)
    np.testing.assert_array_equal(y32.astype(np.float16), y16)
    ys32 = y32 if x.ndim == 2 else y32[None, :]
    ys16 = y16 if x.ndim == 2 else y16[None, :]
    for b in range(xs.shape[0]):
        check_parity(ys32[b], y_ref[b], xs[b], bound, f32_out=True)
        check_parity(ys16[b], y_ref[b], xs[b], bound)
    np.testing.assert_array_equal(run(p, x, f32_out=True, shared=shared), y32)   # bitwise reproducible
    return y32


# m, n, q, g, mode, shared-scale layout
GEMV_CASES = [
    (48, 131072, 3, 128, "greedy", False),     # the plain case
    (48, 131072, 3, 128, "rtn", False),        # offsets (eq. 3) carried across tiles
    (48, 131072, 5, 128, "greedy_z", False),   # more than four planes
    (33, 131072, 8, 0, "greedy", False),       # eight planes, row-wise scales, ragged rows
    (48, 131072, 3, 32, "rtn", False),         # one scale set per pair of slots
    (48, 147456, 4, 96, "greedy_z", False),    # ... with groups of 96 columns, which straddle K tiles
    (48, 131872, 5, 32, "rtn", False),         # ... five planes, last tile of 100 chunks
    (48, 131072, 2, 32, "rtn", True),          # ... shared-scale layout
    (48, 131072, 3, 16, "rtn", False),         # one scale set per slot
    (48, 147456, 2, 24, "greedy_z", False),    # g = 8 * 3: one scale set per chunk
    (48, 131072, 3, 64, "rtn", True),          # shared-scale layout
    (20, 131592, 2, 8, "rtn", True),           # shared scales, per-chunk sets, last tile of 65 chunks
    (6400, 20480, 3, 128, "greedy_z", False),  # many row ranges, several rounds of units per tile
    (640, 98304, 4, 128, "greedy", False),
]


@pytest.mark.parametrize("m,n,q,g,mode,shared", GEMV_CASES)
def test_gemv_several_tiles_per_k_group(m, n, q, g, mode, shared):
    kg, tpg, rs = L.lutgemm_plan_grid(m, n, q, g, 1)
    print(f"case gemv m={m} n={n} q={q} g={g} mode={mode} shared={shared}: grid KG={kg} TPG={tpg} RS={rs}", flush=True)
    assert tpg > 1, "this shape is meant to reach K groups of several tiles"
    W = synth.weights_fp16(m, n, seed=11000 + m + q)
    x = synth.activations_fp16(n, seed=11500 + m + q)
    p = Packed.from_weights(W, q, g, MODES[mode])
    del W
    if shared:
        p.share()
        y_planes = run(p, x, f32_out=True)
        np.testing.assert_array_equal(run(p, x, f32_out=True, shared=True), y_planes)
    _check_all_rows(p, x, shared=False)


# m, n, q, g, mode, batch, kernel width the case is about (2: pair kernel, 4: quad kernel)
BATCH_CASES = [
    (40, 65536, 3, 128, "greedy", 2, 2),
    (640, 40960, 3, 128, "rtn", 2, 2),         # offsets, several row ranges
    (640, 40960, 6, 128, "greedy_z", 2, 2),    # more than four planes
    (300, 49152, 3, 32, "rtn", 2, 2),          # one scale set per slot
    (200, 65536, 2, 8, "greedy_z", 2, 2),      # smallest groups
    (640, 40960, 3, 128, "rtn", 4, 4),
    (640, 40960, 5, 128, "greedy_z", 3, 4),    # three vectors through the quad kernel, five planes
    (300, 49152, 4, 32, "rtn", 4, 4),
    (333, 41480, 2, 8, "greedy", 4, 4),        # ragged rows, last tile of 65 chunks
    (1000, 32768, 3, 128, "greedy", 7, 4),     # 4 + 2 + 1: all three kernels on one layer
]


@pytest.mark.parametrize("m,n,q,g,mode,batch,width", BATCH_CASES)
def test_small_batch_several_tiles_per_k_group(m, n, q, g, mode, batch, width):
    kg, tpg, rs = L.lutgemm_plan_grid(m, n, q, g, width)
    print(f"case batch m={m} n={n} q={q} g={g} mode={mode} batch={batch}: width {width} grid KG={kg} TPG={tpg} RS={rs}",
          flush=True)
    assert tpg > 1, "this shape is meant to reach K groups of several (half, quarter) tiles"
    W = synth.weights_fp16(m, n, seed=12000 + m + q)
    X = synth.activations_fp16(n, seed=12500 + m + q, batch=batch)
    p = Packed.from_weights(W, q, g, MODES[mode])
    del W
    _check_all_rows(p, X)


# K groups that run from tiles of two sub-slabs into a last tile of one (the two kinds of
# tile are walked by different instantiations of the same code, one after the other, on
# the same running sums).  m, n, q, g, mode, batch, kernel width
MIXED_TILE_CASES = [
    (640, 20736, 3, 128, "greedy_z", 4, 4),    # 20 tiles + 256 columns; three quarters per K group
    (2000, 44288, 3, 128, "greedy", 2, 2),     # 43 tiles + 256 columns; three half tiles per K group
]


@pytest.mark.parametrize("m,n,q,g,mode,batch,width", MIXED_TILE_CASES)
def test_small_batch_k_group_across_tile_kinds(m, n, q, g, mode, batch, width):
    kg, tpg, rs = L.lutgemm_plan_grid(m, n, q, g, width)
    tiles = (n // 8 + 127) // 128
    assert 0 < n // 8 - 128 * (tiles - 1) <= 64, "the last tile is meant to have one sub-slab"
    first_of_last_tile = (tiles - 1) * width
    print(f"case mixed m={m} n={n} q={q} g={g} mode={mode} batch={batch}: width {width} grid KG={kg} TPG={tpg} RS={rs}",
          flush=True)
    assert first_of_last_tile % tpg != 0, "a K group is meant to start before the last tile and end in it"
    W = synth.weights_fp16(m, n, seed=14000 + n + q)
    X = synth.activations_fp16(n, seed=14500 + n + q, batch=batch)
    p = Packed.from_weights(W, q, g, MODES[mode])
    del W
    _check_all_rows(p, X)


# Row ranges longer than the running sums in LDS cover (240 row blocks for two vectors, 120
# for four): the workgroup walks its range in stretches, each over all the (half, quarter)
# tiles of its K group.  m, n, q, g, mode, batch, kernel width
LONG_RANGE_CASES = [
    (1000000, 72, 3, 8, "rtn", 2, 2),          # one half tile, two stretches
    (1000000, 72, 3, 8, "rtn", 3, 4),          # one quarter, several stretches, three vectors
    (130000, 1096, 3, 0, "greedy_z", 4, 4),    # two quarters per K group, one K group of quarters that do not exist
    (65536, 16384, 2, 128, "greedy", 2, 2),    # two half tiles per K group, two stretches
    (65536, 16384, 2, 128, "greedy", 4, 4),    # eight quarters per K group, two stretches
]


@pytest.mark.parametrize("m,n,q,g,mode,batch,width", LONG_RANGE_CASES)
def test_small_batch_long_row_ranges(m, n, q, g, mode, batch, width):
    kg, tpg, rs = L.lutgemm_plan_grid(m, n, q, g, width)
    rb = (m + 15) // 16
    blocks = -(-rb // rs) if width == 2 else 2 * -(-((rb + 1) // 2) // rs)
    print(f"case long m={m} n={n} q={q} g={g} mode={mode} batch={batch}: width {width} grid KG={kg} TPG={tpg} RS={rs}, "
          f"{blocks} row blocks per range", flush=True)
    assert blocks > (240 if width == 2 else 120), "this shape is meant to reach row ranges of several stretches"
    W = synth.weights_fp16(m, n, seed=13000 + n + q)
    X = synth.activations_fp16(n, seed=13500 + n + q, batch=batch)
    p = Packed.from_weights(W, q, g, MODES[mode])
    del W
    _check_all_rows(p, X)


def test_plan_grid_reports_what_is_launched():
    # the OPT-175B layers on this device: several tiles per K group on FC2 (n = 49152), one on
    # the out projection; workgroups never exceed the compute units
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for name, (m, n) in synth.OPT_175B.items():
        for width in (1, 2, 4):
            kg, tpg, rs = L.lutgemm_plan_grid(m, n, 3, 128, width)
            tiles = ((n // 8 + 127) // 128) * width
            assert kg * tpg >= tiles and (kg - 1) * tpg < tiles
            assert kg * rs <= max(cus, kg)
    assert L.lutgemm_plan_grid(*synth.OPT_175B["fc2"], 3, 128, 1)[1] > 1
    assert L.lutgemm_plan_grid(*synth.OPT_175B["out"], 3, 128, 1)[1] == 1


@pytest.mark.parametrize("m,n,q,g,batch", [(4096, 16384, 3, 128, 1), (2048, 32768, 3, 128, 1), (4096, 16384, 3, 128, 4)])
def test_split_k_hand_off_over_many_launches(m, n, q, g, batch):
    """The cross-group reduction (partials, arrival counter, last workgroup sums) must give the
    same bits on every one of several hundred back-to-back launches that share one workspace,
    while another stream keeps the memory system busy, and those bits must be the oracle's."""
    from gpu_util import make_workspace, torch_cuda
    torch = torch_cuda()
    kg, tpg, rs = L.lutgemm_plan_grid(m, n, q, g, batch)
    print(f"case hand-off m={m} n={n} q={q} g={g} batch={batch}: grid KG={kg} TPG={tpg} RS={rs}", flush=True)
    assert kg > 1, "this shape is meant to have several K groups"
    W = synth.weights_fp16(m, n, seed=13000 + n + batch)
    p = Packed.from_weights(W, q, g)
    del W
    X = np.stack([synth.activations_fp16(n, seed=13500 + b) for b in range(batch)])
    x = X[0] if batch == 1 else X
    y_first = _check_all_rows(p, x)

    launches = 300
    d_x = torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda()
    d_y = torch.full((launches, batch, m), float("nan"), dtype=torch.float32, device="cuda")
    wsb = L.lutgemm_workspace_bytes(m, n, q, g, 8, batch)
    d_ws = make_workspace(wsb)
    side = torch.cuda.Stream()
    a = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    s = torch.cuda.current_stream()
    torch.cuda.synchronize()
    for i in range(launches):
        if i % 10 == 0:
            with torch.cuda.stream(side):
                b.copy_(a, non_blocking=True)
        if batch == 1:
            L.lutgemm_gemv(d_x, p.d_bits, p.d_alpha, p.d_z, d_y[i], q, g, 8, m, n, L.LUTGEMM_Y_F32, d_ws, wsb, s.cuda_stream)
        else:
            L.lutgemm_gemm(d_x, p.d_bits, p.d_alpha, p.d_z, d_y[i], q, g, 8, m, n, batch, L.LUTGEMM_Y_F32, d_ws, wsb,
                           s.cuda_stream)
    torch.cuda.synchronize()
    want = torch.from_numpy(np.ascontiguousarray(y_first).reshape(1, batch, m)).cuda()
    same = (d_y == want).all(dim=2).all(dim=1)
    assert bool(same.all()), f"launches that differ from the first: {(~same).nonzero().flatten().tolist()[:10]}"
