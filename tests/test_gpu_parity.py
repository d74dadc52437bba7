"""GPU parity: lutgemm_gemv / lutgemm_gemm through the C ABI against the fp64 oracle,
element by element, on seeded inputs spanning several tiles, ragged tails and the
degenerate cases of the format."""
import numpy as np
import pytest

import paper_2206_09557_amd as L
from oracle import bcq_oracle as O
from oracle import c_oracle
from paper_2206_09557_amd import synth

from gpu_util import Packed, check_parity, make_workspace, row_l1_bound, run

pytestmark = pytest.mark.gpu

MODES = {"greedy": L.LUTGEMM_Q_GREEDY, "greedy_z": L.LUTGEMM_Q_GREEDY_MEAN_OFFSET, "rtn": L.LUTGEMM_Q_UNIFORM_RTN,
         "alt": L.LUTGEMM_Q_ALTERNATING}


def _oracle_full(p, x16):
    """fp64 y from the packed host buffers, numpy oracle (own decoder + definition)."""
    return O.gemv_packed(p.bits, p.alpha, p.z, x16, p.m, p.n, p.q, p.g)


def _bound(p):
    g = p.n if p.g == 0 else p.g
    NG = p.n // g
    a = O.decode_alpha(p.alpha, p.m, NG, p.q)
    z = None if p.z is None else O.decode_z(p.z, p.m, NG)
    return row_l1_bound(a, z, g)


# m, n, q, g, mode -- config 1 of the workload list first, then ragged / degenerate shapes
CASES = [
    (1024, 1024, 3, 128, "greedy"),      # single GEMV m = n = 1024, q = 3, g = 128, no offset
    (50, 1544, 2, 8, "greedy_z"),        # ragged rows, last tile with 65 chunks, g = 8 (pair spans two groups)
    (1000, 1536, 4, 128, "greedy_z"),    # last tile with exactly 64 chunks (one sub-slab)
    (77, 520, 3, 0, "greedy"),           # single ragged tile, row-wise scales
    (300, 2048, 3, 32, "rtn"),           # uniform -> BCQ with offset, small groups
    (300, 2048, 2, 64, "rtn"),
    (1, 8, 1, 8, "greedy"),              # smallest legal problem
    (16, 8, 8, 8, "rtn"),
    (4100, 3072, 3, 128, "greedy"),      # several workgroups per tile, ragged split of row blocks
    (515, 5120, 4, 128, "greedy"),
    (130, 1032, 5, 24, "greedy_z"),      # g % 16 != 0, second tile holds one chunk
    (96, 1048, 3, 8, "rtn"),             # ragged tile AND split groups
    (200, 1024, 3, 128, "alt"),          # alternating BCQ scales (not ordered by plane)
    (130, 1000, 6, 40, "greedy_z"),      # single ragged tile (y written without the cross-group pass), q > 4
]


@pytest.mark.parametrize("m,n,q,g,mode", CASES)
def test_gemv_matches_oracle(m, n, q, g, mode):
    print(f"case m={m} n={n} q={q} g={g} mode={mode}", flush=True)
    W = synth.weights_fp16(m, n, seed=1000 + m + 7 * n + q)
    x = synth.activations_fp16(n, seed=1500 + m + n)
    p = Packed.from_weights(W, q, g, MODES[mode])
    y_ref = _oracle_full(p, x)
    bound = _bound(p)
    y16 = run(p, x)
    check_parity(y16, y_ref, x, bound)
    y32 = run(p, x, f32_out=True)
    check_parity(y32, y_ref, x, bound, f32_out=True)
    # fp16 output is the single rounding of the fp32 result
    np.testing.assert_array_equal(y32.astype(np.float16), y16)
    # bitwise reproducible
    np.testing.assert_array_equal(run(p, x, f32_out=True), y32)


@pytest.mark.parametrize("q", range(1, 9))
def test_every_q(q):
    print(f"case q={q}", flush=True)
    m, n, g = 200, 2560, 128
    W = synth.weights_fp16(m, n, seed=2000 + q)
    x = synth.activations_fp16(n, seed=2500 + q)
    for mode in ("greedy", "rtn"):
        p = Packed.from_weights(W, q, g, MODES[mode])
        check_parity(run(p, x, f32_out=True), _oracle_full(p, x), x, _bound(p), f32_out=True)


@pytest.mark.parametrize("n", [2048, 1024])   # 1024: a single tile, the left-over vector's y is written directly
@pytest.mark.parametrize("batch", [1, 2, 5, 32])
def test_gemm_batches(batch, n):
    print(f"case batch={batch} n={n}", flush=True)
    m, q, g = 333, 3, 128
    W = synth.weights_fp16(m, n, seed=3000)
    X = synth.activations_fp16(n, seed=3500 + batch, batch=batch)
    for mode in ("greedy", "greedy_z"):
        p = Packed.from_weights(W, q, g, MODES[mode])
        Y = run(p, X, f32_out=True)
        assert Y.shape == (batch, m)
        bound = _bound(p)
        for b in range(batch):
            check_parity(Y[b], _oracle_full(p, X[b]), X[b], bound, f32_out=True)
        Y16 = run(p, X)
        np.testing.assert_array_equal(Y.astype(np.float16), Y16)


def test_known_planes_unit_scale_signed_sum():
    # q = 1, alpha = 1, z = 0: y_r = sum_k +-x_k, planes given directly (no quantiser)
    rng = np.random.default_rng(4000)
    m, n = 70, 1032
    B = rng.choice(np.array([-1, 1], dtype=np.int8), size=(1, m, n))
    B[0, 0, :] = 1
    B[0, 1, :] = -1
    bits = L.lutgemm_pack_planes(B)
    ap, _ = L.lutgemm_pack_scales(np.ones((1, m, 1), dtype=np.float16), None, n, 0)
    x = synth.activations_fp16(n, seed=4001)
    p = Packed(bits, ap, None, m, n, 1, 0)
    y = run(p, x, f32_out=True)
    want = B[0].astype(np.float64) @ x.astype(np.float64)
    np.testing.assert_allclose(y, want, rtol=0, atol=2e-4)
    assert abs(y[0] + y[1]) < 1e-6


def test_special_values_in_x():
    # zeros, the largest finite fp16 scaled so that sums stay finite, subnormals
    m, n, q, g = 64, 1024, 2, 128
    W = synth.weights_fp16(m, n, seed=4100)
    p = Packed.from_weights(W, q, g)
    x = np.zeros(n, dtype=np.float16)
    assert np.all(run(p, x, f32_out=True) == 0)
    x = synth.activations_fp16(n, seed=4101)
    x[::3] = 0
    x[1::97] = np.float16(6.0e-8)       # subnormal
    x[5::101] = np.float16(2048.0)
    check_parity(run(p, x, f32_out=True), _oracle_full(p, x), x, _bound(p), f32_out=True)


def test_one_workspace_serves_many_calls_and_shapes():
    # the arrival counters are left at zero by every call: a workspace prepared once is
    # reused across calls, shapes, batch sizes and output types
    ws = make_workspace(L.lutgemm_workspace_bytes(4100, 3072, 3, 128, 8, 4))
    for (m, n, q, g, batch) in [(4100, 3072, 3, 128, None), (515, 2048, 2, 64, None), (4100, 3072, 3, 128, 4),
                                (77, 520, 3, 0, None), (4100, 3072, 3, 128, None)]:
        print(f"case m={m} n={n} q={q} g={g} batch={batch}", flush=True)
        W = synth.weights_fp16(m, n, seed=4300 + m)
        x = synth.activations_fp16(n, seed=4301 + m, batch=batch)
        p = Packed.from_weights(W, q, g)
        y = run(p, x, f32_out=True, workspace=ws)
        np.testing.assert_array_equal(y, run(p, x, f32_out=True))
        np.testing.assert_array_equal(y, run(p, x, f32_out=True, workspace=ws))


def test_runs_on_a_side_stream():
    torch = pytest.importorskip("torch")
    m, n, q, g = 512, 2048, 3, 128
    W = synth.weights_fp16(m, n, seed=4200)
    x = synth.activations_fp16(n, seed=4201)
    p = Packed.from_weights(W, q, g)
    s = torch.cuda.Stream()
    y_side = run(p, x, f32_out=True, stream=s)
    np.testing.assert_array_equal(y_side, run(p, x, f32_out=True))


# ---- matrix-core path (lutgemm_gemm_mfma): same oracle, same tolerances ----

MFMA_CASES = [
    (1024, 1024, 3, 128, "greedy", 4),
    (333, 2048, 3, 128, "greedy_z", 5),     # ragged rows, offsets
    (1000, 1536, 4, 128, "greedy_z", 16),   # last tile with exactly 64 chunks (one sub-slab)
    (77, 576, 3, 0, "greedy", 1),           # single ragged tile, row-wise scales, one vector
    (300, 2048, 2, 64, "rtn", 17),          # smallest supported group, more than 16 vectors
    (4100, 3072, 3, 128, "greedy", 32),     # several workgroups, ragged split of row blocks, full batch
    (515, 5120, 4, 128, "greedy", 2),
    (130, 4224, 5, 192, "greedy_z", 3),     # q > 4 (4-wavefront workgroups), groups that straddle K tiles
    (96, 1088, 8, 64, "rtn", 20),           # eight planes, ragged last tile of 8 chunks
    (16, 64, 1, 64, "greedy", 32),          # smallest supported problem
]


@pytest.mark.parametrize("m,n,q,g,mode,batch", MFMA_CASES)
def test_mfma_path_matches_oracle(m, n, q, g, mode, batch):
    print(f"case mfma m={m} n={n} q={q} g={g} mode={mode} batch={batch}", flush=True)
    W = synth.weights_fp16(m, n, seed=6000 + m + 7 * n + q)
    X = synth.activations_fp16(n, seed=6500 + m + n, batch=batch)
    p = Packed.from_weights(W, q, g, MODES[mode])
    bound = _bound(p)
    Y32 = run(p, X, f32_out=True, mfma=True)
    assert Y32.shape == (batch, m)
    for b in range(batch):
        check_parity(Y32[b], _oracle_full(p, X[b]), X[b], bound, f32_out=True)
    Y16 = run(p, X, mfma=True)
    np.testing.assert_array_equal(Y32.astype(np.float16), Y16)
    np.testing.assert_array_equal(run(p, X, f32_out=True, mfma=True), Y32)   # bitwise reproducible


@pytest.mark.parametrize("m,n,q,g,mode,batch", MFMA_CASES)
def test_dequant_mfma_kernel_matches_oracle_to_fp16_weight_rounding(m, n, q, g, mode, batch):
    # the dequantise-then-multiply comparison kernel: same oracle; its method rounds the rebuilt
    # weights to fp16, so it is held to relative L2 <= 1e-3 and the row-L1 bound, not to 1e-5
    print(f"case dequant m={m} n={n} q={q} g={g} mode={mode} batch={batch}", flush=True)
    W = synth.weights_fp16(m, n, seed=6000 + m + 7 * n + q)
    X = synth.activations_fp16(n, seed=6500 + m + n, batch=batch)
    p = Packed.from_weights(W, q, g, MODES[mode])
    bound = _bound(p)
    Y32 = run(p, X, f32_out=True, dequant=True)
    assert Y32.shape == (batch, m)
    worst = 0.0
    for b in range(batch):
        worst = max(worst, check_parity(Y32[b], _oracle_full(p, X[b]), X[b], bound, f32_out=True, fp16_weights=True))
    print(f"worst relative L2 {worst:.2e}", flush=True)
    np.testing.assert_array_equal(Y32.astype(np.float16), run(p, X, dequant=True))
    np.testing.assert_array_equal(run(p, X, f32_out=True, dequant=True), Y32)   # bitwise reproducible
    # and it is a different computation from the plane-wise path, not an alias of it
    if q > 1:
        assert not np.array_equal(Y32, run(p, X, f32_out=True, mfma=True))


def test_mfma_path_rejects_groups_not_multiple_of_64():
    m, n, q, g = 64, 1024, 2, 32
    W = synth.weights_fp16(m, n, seed=6900)
    p = Packed.from_weights(W, q, g)
    X = synth.activations_fp16(n, seed=6901, batch=2)
    with pytest.raises(L.LutGemmError) as e:
        run(p, X, mfma=True)
    assert e.value.code == L.LUTGEMM_EUNSUPPORTED


# ---- shared-scale layout (one scale per group, appendix C) ----

def test_auto_path_is_one_of_the_two():
    # LUTGEMM_PATH_AUTO: by shape and batch alone, the matrix-core path from five vectors on
    # (three on small layers) where it applies, else the lookup path; bit for bit that path's y
    m, n, q = 300, 2048, 3
    W = synth.weights_fp16(m, n, seed=5600)
    for g, batch, want_mfma in [(128, 8, True), (128, 5, True), (128, 4, True), (128, 3, True), (128, 2, False),
                                (128, 1, False), (32, 8, False), (0, 6, True)]:
        print(f"case g={g} batch={batch}", flush=True)
        p = Packed.from_weights(W, q, g, MODES["greedy_z"])
        X = synth.activations_fp16(n, seed=5601 + batch, batch=batch)
        y_auto = run(p, X, f32_out=True, auto=True)
        y_want = run(p, X, f32_out=True, mfma=want_mfma)
        np.testing.assert_array_equal(y_auto, y_want)
        for b in range(batch):
            check_parity(y_auto[b], _oracle_full(p, X[b]), X[b], _bound(p), f32_out=True)
    # shared scales: always the lookup path
    p = Packed.from_weights(W, q, 128, MODES["rtn"]).share()
    X = synth.activations_fp16(n, seed=5610, batch=8)
    np.testing.assert_array_equal(run(p, X, f32_out=True, auto=True, shared=True), run(p, X, f32_out=True, shared=True))


SHARED_CASES = [
    (300, 2048, 3, 32, None),     # small groups: the scale bytes matter most here
    (300, 2048, 2, 64, None),
    (1000, 1536, 4, 128, None),   # last tile with one sub-slab
    (96, 1048, 3, 8, None),       # per-chunk scale fetches, ragged tile
    (130, 1032, 5, 24, None),     # more than four planes, a scale set per chunk (fetched plane by plane)
    (77, 520, 8, 0, None),        # row-wise, eight planes
    (4100, 3072, 3, 128, 5),      # batch: pairs and an odd last vector
    (333, 2048, 4, 32, 2),
]


@pytest.mark.parametrize("m,n,q,g,batch", SHARED_CASES)
def test_shared_scales_equal_per_plane_scales_bitwise(m, n, q, g, batch):
    print(f"case shared m={m} n={n} q={q} g={g} batch={batch}", flush=True)
    W = synth.weights_fp16(m, n, seed=7000 + m + 7 * n + q)
    x = synth.activations_fp16(n, seed=7500 + m + n, batch=batch)
    p = Packed.from_weights(W, q, g, L.LUTGEMM_Q_UNIFORM_RTN).share()
    y_planes = run(p, x, f32_out=True)
    y_shared = run(p, x, f32_out=True, shared=True)
    np.testing.assert_array_equal(y_shared, y_planes)
    np.testing.assert_array_equal(run(p, x, shared=True), run(p, x))
    # and against the oracle reading the shared layout itself
    bound = _bound(p)
    xs = x if batch else x[None, :]
    ys = y_shared if batch else y_shared[None, :]
    for b in range(xs.shape[0]):
        y_ref = O.gemv_packed(p.bits, p.alpha_shared, p.z, xs[b], m, n, q, g, alpha_shared=True)
        check_parity(ys[b], y_ref, xs[b], bound, f32_out=True)


def test_shared_scales_need_offsets():
    m, n, q, g = 64, 1024, 2, 64
    W = synth.weights_fp16(m, n, seed=7900)
    p = Packed.from_weights(W, q, g, L.LUTGEMM_Q_UNIFORM_RTN).share()
    p.d_z = None
    with pytest.raises(L.LutGemmError) as e:
        run(p, synth.activations_fp16(n, seed=7901), shared=True)
    assert e.value.code == L.LUTGEMM_EINVAL


# ---- seeded sweep over random small shapes: every path against the oracle ----

def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        q = int(rng.integers(1, 9))
        g_units = int(rng.choice([1, 2, 3, 4, 8, 16, 24]))          # group size in chunks of 8 columns
        groups = int(rng.integers(1, 40))
        n = 8 * g_units * groups
        if n > 4096:
            continue
        g = 0 if rng.random() < 0.15 else 8 * g_units
        m = int(rng.integers(1, 400))
        mode = ["greedy", "greedy_z", "rtn"][int(rng.integers(0, 3))]
        batch = [None, None, 2, 3, 7, 18][int(rng.integers(0, 6))]
        cases.append((m, n, q, g, mode, batch))
    return cases


@pytest.mark.parametrize("m,n,q,g,mode,batch", _random_cases(36, 20240607))
def test_random_shapes_all_paths(m, n, q, g, mode, batch):
    print(f"case random m={m} n={n} q={q} g={g} mode={mode} batch={batch}", flush=True)
    W = synth.weights_fp16(m, n, seed=8000 + m + 3 * n + q)
    x = synth.activations_fp16(n, seed=8500 + m + n, batch=batch)
    p = Packed.from_weights(W, q, g, MODES[mode])
    bound = _bound(p)
    xs = x if batch else x[None, :]
    refs = [_oracle_full(p, xs[b]) for b in range(xs.shape[0])]

    def check(y):
        ys = y if batch else y[None, :]
        for b in range(xs.shape[0]):
            check_parity(ys[b], refs[b], xs[b], bound, f32_out=True)

    y = run(p, x, f32_out=True)
    check(y)
    gg = n if g == 0 else g
    if gg % 64 == 0:                       # the matrix-core path takes these group sizes only
        ym = run(p, xs, f32_out=True, mfma=True)
        for b in range(xs.shape[0]):
            check_parity(ym[b], refs[b], xs[b], bound, f32_out=True)
    if mode == "rtn":                      # shared-scale layout: bitwise the same as per-plane scales
        p.share()
        np.testing.assert_array_equal(run(p, x, f32_out=True, shared=True), y)


def _random_wide_cases(count, seed):
    """Long rows, few of them, small batches: K groups of several (half, quarter) tiles in the
    pair and quad kernels, ragged last tiles of either kind, every scale mode."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        q = int(rng.integers(1, 9))
        g_units = int(rng.choice([1, 2, 3, 4, 8, 16, 24]))
        groups = int(rng.integers(40, 1200))
        n = 8 * g_units * groups
        if n < 6144 or n > 70000:
            continue
        g = 0 if rng.random() < 0.15 else 8 * g_units
        m = int(rng.integers(1, 600))
        mode = ["greedy", "greedy_z", "rtn"][int(rng.integers(0, 3))]
        batch = [2, 3, 4, 6, 7][int(rng.integers(0, 5))]
        cases.append((m, n, q, g, mode, batch))
    return cases


@pytest.mark.parametrize("m,n,q,g,mode,batch", _random_wide_cases(24, 20240611))
def test_random_wide_shapes_small_batch(m, n, q, g, mode, batch):
    grids = [L.lutgemm_plan_grid(m, n, q, g, width) for width in (1, 2, 4)]
    print(f"case wide m={m} n={n} q={q} g={g} mode={mode} batch={batch} grids (KG, TPG, RS) {grids}", flush=True)
    W = synth.weights_fp16(m, n, seed=9000 + m + 3 * n + q)
    X = synth.activations_fp16(n, seed=9500 + m + n, batch=batch)
    p = Packed.from_weights(W, q, g, MODES[mode])
    del W
    bound = _bound(p)
    y_ref, _ = c_oracle.gemv_packed(p.bits, p.alpha, p.z, X, p.m, p.n, p.q, p.g)
    y = run(p, X, f32_out=True)
    for b in range(batch):
        check_parity(y[b], y_ref[b], X[b], bound, f32_out=True)
    np.testing.assert_array_equal(run(p, X, f32_out=True), y)    # bitwise reproducible
    if mode == "rtn":                      # shared-scale layout: bitwise the same as per-plane scales
        p.share()
        np.testing.assert_array_equal(run(p, X, f32_out=True, shared=True), y)


def _random_wide_gemv_cases(count, seed):
    """Long rows at batch 1: K groups of several tiles in the GEMV kernel with every plane count
    and every scale mode, group sizes that are odd multiples of 32 columns among them (one scale
    set per pair of slots), ragged last tiles of either kind."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        q = int(rng.integers(1, 9))
        g_units = int(rng.choice([1, 2, 3, 4, 4, 8, 12, 12, 16, 20, 24]))
        m = int(rng.integers(1, 100)) if rng.random() < 0.6 else int(rng.integers(100, 900))
        groups = int(rng.integers(40, 6000))
        n = 8 * g_units * groups
        if n < 6144 or n > (300000 if m < 100 else 70000):   # few rows, very long: several tiles per K group
            continue
        g = 0 if rng.random() < 0.1 else 8 * g_units
        mode = ["greedy", "greedy_z", "rtn"][int(rng.integers(0, 3))]
        cases.append((m, n, q, g, mode))
    return cases


@pytest.mark.parametrize("m,n,q,g,mode", _random_wide_gemv_cases(20, 20240613))
def test_random_wide_shapes_gemv(m, n, q, g, mode):
    print(f"case wide gemv m={m} n={n} q={q} g={g} mode={mode} grid (KG, TPG, RS) {L.lutgemm_plan_grid(m, n, q, g, 1)}",
          flush=True)
    W = synth.weights_fp16(m, n, seed=9700 + m + 3 * n + q)
    x = synth.activations_fp16(n, seed=9800 + m + n)
    p = Packed.from_weights(W, q, g, MODES[mode])
    del W
    bound = _bound(p)
    y_ref, _ = c_oracle.gemv_packed(p.bits, p.alpha, p.z, x[None, :], p.m, p.n, p.q, p.g)
    y = run(p, x, f32_out=True)
    check_parity(y, y_ref[0], x, bound, f32_out=True)
    check_parity(run(p, x), y_ref[0], x, bound)
    np.testing.assert_array_equal(run(p, x, f32_out=True), y)    # bitwise reproducible
    if mode == "rtn":                      # shared-scale layout: bitwise the same as per-plane scales
        p.share()
        np.testing.assert_array_equal(run(p, x, f32_out=True, shared=True), y)


@pytest.mark.parametrize("m,n,q,g,batch", [
    (16, 262144, 2, 128, None),     # one row block, 256 K tiles: deep split-K
    (40, 65536, 3, 1024, 4),        # few rows, long rows, four vectors
    (200000, 64, 2, 64, None),      # many rows, a single ragged K tile of 8 chunks
    (70001, 128, 3, 0, 6),          # odd number of row blocks, row-wise scales, 4 + 2 vectors
])
def test_extreme_aspect_ratios(m, n, q, g, batch):
    print(f"case extreme m={m} n={n} q={q} g={g} batch={batch}", flush=True)
    W = synth.weights_fp16(m, n, seed=9000 + q)
    x = synth.activations_fp16(n, seed=9500 + q, batch=batch)
    p = Packed.from_weights(W, q, g)
    del W
    rows = np.unique(np.concatenate([np.arange(min(m, 40)), np.arange(max(0, m - 40), m),
                                     np.random.default_rng(9).integers(0, m, size=60)]))
    a = O.decode_alpha(p.alpha, m, 1 if g == 0 else n // g, q)
    bound = row_l1_bound(a, None, n if g == 0 else g)
    y = run(p, x, f32_out=True)
    xs = x if batch else x[None, :]
    ys = y if batch else y[None, :]
    yref, _ = c_oracle.gemv_packed(p.bits, p.alpha, None, xs, m, n, q, g, rows=rows)
    for b in range(xs.shape[0]):
        check_parity(ys[b][rows], yref[b], xs[b], bound[rows], f32_out=True)
    if (n if g == 0 else g) % 64 == 0:
        ym = run(p, xs, f32_out=True, mfma=True)
        for b in range(xs.shape[0]):
            check_parity(ym[b][rows], yref[b], xs[b], bound[rows], f32_out=True)


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    # serving loops replay captured work: the entry points enqueue kernels only (no allocation,
    # no synchronisation, counters reset by the kernels themselves), so a captured call must
    # give the eager result on every replay, also after the inputs have changed in place
    import torch
    m, n, q, g, batch = 1500, 3072, 3, 128, 7          # 4 + 2 + 1 vectors: all three lookup kernels
    W = synth.weights_fp16(m, n, seed=9900)
    p = Packed.from_weights(W, q, g)
    wsb = L.lutgemm_workspace_bytes(m, n, q, g, 8, batch)
    ws = make_workspace(wsb)
    d_x = torch.zeros((batch, n), dtype=torch.float16, device="cuda")
    d_y = torch.zeros((batch, m), dtype=torch.float32, device="cuda")
    d_y1 = torch.zeros(m, dtype=torch.float32, device="cuda")
    d_ym = torch.zeros((batch, m), dtype=torch.float32, device="cuda")
    ws2, ws3 = make_workspace(wsb), make_workspace(wsb)

    def enqueue(stream):
        L.lutgemm_gemm(d_x, p.d_bits, p.d_alpha, None, d_y, q, g, 8, m, n, batch, L.LUTGEMM_Y_F32, ws, wsb, stream)
        L.lutgemm_gemv(d_x, p.d_bits, p.d_alpha, None, d_y1, q, g, 8, m, n, L.LUTGEMM_Y_F32, ws2, wsb, stream)
        L.lutgemm_gemm_mfma(d_x, p.d_bits, p.d_alpha, None, d_ym, q, g, 8, m, n, batch, L.LUTGEMM_Y_F32, ws3, wsb, stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        enqueue(side.cuda_stream)                       # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for rep in range(3):
        x = synth.activations_fp16(n, seed=9910 + rep, batch=batch)
        d_x.copy_(torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16))
        d_y.fill_(float("nan")); d_y1.fill_(float("nan")); d_ym.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, got1, gotm = d_y.cpu().numpy(), d_y1.cpu().numpy(), d_ym.cpu().numpy()
        np.testing.assert_array_equal(got, run(p, x, f32_out=True))
        np.testing.assert_array_equal(got1, run(p, x[0], f32_out=True))
        np.testing.assert_array_equal(gotm, run(p, x, f32_out=True, mfma=True))
