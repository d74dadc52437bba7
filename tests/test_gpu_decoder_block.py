"""GPU parity of the decoder-layer sequence (the four linear layers of a decoder block, paper
appendix A) at the OPT-175B shapes, q = 3, g = 128: once as four lutgemm_gemv calls enqueued
back to back on one stream with ONE shared workspace and a single synchronisation at the end,
once as one lutgemm_gemv_group launch.  All four outputs, every row, against the fp64 C oracle;
the grouped launch must equal the four calls bit for bit.  Smaller groups cover offsets, shared
scales, mixed shapes with row-wise scales and the refusals."""
import numpy as np
import pytest

import paper_2206_09557_amd as L
from oracle import bcq_oracle as O
from oracle import c_oracle
from paper_2206_09557_amd import synth

from gpu_util import Packed, check_parity, make_workspace, row_l1_bound, torch_cuda

pytestmark = pytest.mark.gpu


def _bounds(p):
    g = p.n if p.g == 0 else p.g
    a = O.decode_alpha(p.alpha, p.m, p.n // g, p.q)
    z = None if p.z is None else O.decode_z(p.z, p.m, p.n // g)
    return row_l1_bound(a, z, g)


def _run_sequence(layers, xs, q, g, f32_out, shared=False):
    """Four (or any number of) lutgemm_gemv calls back to back, one workspace, one sync."""
    torch = torch_cuda()
    flags = (L.LUTGEMM_Y_F32 if f32_out else L.LUTGEMM_Y_F16) | (L.LUTGEMM_ALPHA_SHARED if shared else 0)
    wsb = max(L.lutgemm_workspace_bytes(p.m, p.n, q, g) for p in layers)
    ws = make_workspace(wsb)
    d_x = [torch.from_numpy(x.view(np.int16)).cuda() for x in xs]
    d_y = [torch.full((p.m,), float("nan"), dtype=torch.float32 if f32_out else torch.float16, device="cuda")
           for p in layers]
    s = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    for p, dx, dy in zip(layers, d_x, d_y):
        L.lutgemm_gemv(dx, p.d_bits, p.d_alpha_shared if shared else p.d_alpha, p.d_z, dy, q, g, 8, p.m, p.n, flags, ws,
                       wsb, s)
    torch.cuda.synchronize()
    return [dy.cpu().numpy() for dy in d_y]


def _run_group(layers, xs, q, g, f32_out, shared=False):
    torch = torch_cuda()
    flags = (L.LUTGEMM_Y_F32 if f32_out else L.LUTGEMM_Y_F16) | (L.LUTGEMM_ALPHA_SHARED if shared else 0)
    ms, ns = [p.m for p in layers], [p.n for p in layers]
    wsb = L.lutgemm_group_workspace_bytes(ms, ns, q, g)
    assert wsb > 0
    ws = make_workspace(wsb)
    d_x = [torch.from_numpy(x.view(np.int16)).cuda() for x in xs]
    d_y = [torch.full((p.m,), float("nan"), dtype=torch.float32 if f32_out else torch.float16, device="cuda")
           for p in layers]
    z = None if layers[0].d_z is None else [p.d_z for p in layers]
    torch.cuda.synchronize()
    L.lutgemm_gemv_group(d_x, [p.d_bits for p in layers], [p.d_alpha_shared if shared else p.d_alpha for p in layers], z,
                         d_y, ms, ns, q, g, 8, flags, ws, wsb, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    first = [dy.cpu().numpy() for dy in d_y]
    # the workspace is left ready: a second launch on it gives the same bits
    for dy in d_y:
        dy.fill_(float("nan"))
    L.lutgemm_gemv_group(d_x, [p.d_bits for p in layers], [p.d_alpha_shared if shared else p.d_alpha for p in layers], z,
                         d_y, ms, ns, q, g, 8, flags, ws, wsb, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for a, dy in zip(first, d_y):
        np.testing.assert_array_equal(a, dy.cpu().numpy())
    return first


def _check(layers, xs, q, g, shared=False):
    refs = [c_oracle.gemv_packed(p.bits, p.alpha, p.z, x, p.m, p.n, q, g)[0] for p, x in zip(layers, xs)]
    print("oracle done", flush=True)
    for f32_out in (True, False):
        seq = _run_sequence(layers, xs, q, g, f32_out, shared)
        grp = _run_group(layers, xs, q, g, f32_out, shared)
        for p, x, ref, ys, yg in zip(layers, xs, refs, seq, grp):
            check_parity(ys, ref, x, _bounds(p), f32_out=f32_out)
            np.testing.assert_array_equal(yg, ys)


def test_opt175b_decoder_block_sequence_and_group_all_rows():
    q, g = 3, 128
    layers, xs = [], []
    for li, name in enumerate(["qkv", "out", "fc1", "fc2"]):
        m, n = synth.OPT_175B[name]
        print(f"case block layer {name} m={m} n={n}", flush=True)
        W = synth.weights_fp16(m, n, seed=14000 + li)
        layers.append(Packed.from_weights(W, q, g))
        del W
        xs.append(synth.activations_fp16(n, seed=14500 + li))
    _check(layers, xs, q, g)


@pytest.mark.parametrize("shapes,q,g,mode,shared", [
    ([(300, 2048), (77, 520), (1000, 1536)], 3, 0, L.LUTGEMM_Q_GREEDY, False),           # row-wise scales, ragged tiles; group sizes 2048, 520 (not a multiple of 16) -> refused, see below
    ([(4100, 3072), (515, 5120), (64, 1024), (1, 128)], 3, 128, L.LUTGEMM_Q_UNIFORM_RTN, False),   # offsets, a direct single-tile layer, one row
    ([(333, 2048), (200, 4096)], 4, 32, L.LUTGEMM_Q_UNIFORM_RTN, True),                   # shared scales, one scale set per slot
    ([(48, 131072), (640, 98304)], 2, 64, L.LUTGEMM_Q_GREEDY_MEAN_OFFSET, False),         # K groups of several tiles
    ([(130, 2560)] * 8, 6, 128, L.LUTGEMM_Q_GREEDY, False),                               # eight layers, six planes
])
def test_small_groups(shapes, q, g, mode, shared):
    print(f"case group shapes={shapes} q={q} g={g} mode={mode} shared={shared}", flush=True)
    layers, xs = [], []
    for li, (m, n) in enumerate(shapes):
        W = synth.weights_fp16(m, n, seed=15000 + 17 * li + m)
        p = Packed.from_weights(W, q, g, mode)
        layers.append(p.share() if shared else p)
        xs.append(synth.activations_fp16(n, seed=15500 + li + n))
    if g == 0 and len({(n % 64 == 0, n % 32 == 0, n % 16 == 0) for _, n in shapes}) > 1:
        # row-wise group sizes of different classes cannot share one kernel
        with pytest.raises(L.LutGemmError) as e:
            _run_group(layers, xs, q, g, True)
        assert e.value.code == L.LUTGEMM_EUNSUPPORTED
        return
    _check(layers, xs, q, g, shared)


def test_group_refusals():
    torch = torch_cuda()
    d = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    ws = make_workspace(L.lutgemm_group_workspace_bytes([64], [1024], 3, 128))
    def call(count, g=128, flags=0):
        L.lutgemm_gemv_group([d] * count, [d] * count, [d] * count, None, [d] * count, [64] * count, [1024] * count, 3, g, 8,
                             flags, ws, ws.numel(), 0)
    with pytest.raises(L.LutGemmError) as e:
        call(9)
    assert e.value.code == L.LUTGEMM_EUNSUPPORTED
    with pytest.raises(L.LutGemmError) as e:
        call(1, g=8)             # a scale set per chunk: not offered in a group
    assert e.value.code == L.LUTGEMM_EUNSUPPORTED
    with pytest.raises(L.LutGemmError) as e:
        call(1, flags=L.LUTGEMM_ALPHA_SHARED)   # shared scales need offsets
    assert e.value.code == L.LUTGEMM_EINVAL
    assert L.lutgemm_group_workspace_bytes([64] * 9, [1024] * 9, 3, 128) == 0
    assert L.lutgemm_group_workspace_bytes([64, 64], [1024, 1024], 3, 128) == 32768 + 2 * 256   # 64 rows x 4 B per layer
