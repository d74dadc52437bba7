"""GPU test of lutgemm_gemv_static, the entry point that allocates nothing: through the C
ABI, two calls in a row on the library's own scratch array, the second on a smaller layer,
each compared bit for bit with lutgemm_gemv on a caller-provided workspace (which the other
tests hold to the oracle's tolerance), and with the oracle."""
import numpy as np
import pytest

import paper_2206_09557_amd as L
from oracle import bcq_oracle as O
from paper_2206_09557_amd import synth

from gpu_util import Packed, check_parity, row_l1_bound, run, torch_cuda

pytestmark = pytest.mark.gpu


def _static(p, x16, f32_out):
    torch = torch_cuda()
    d_x = torch.from_numpy(np.ascontiguousarray(x16).view(np.int16)).cuda()
    d_y = torch.full((p.m,), float("nan"), dtype=torch.float32 if f32_out else torch.float16, device="cuda")
    flags = L.LUTGEMM_Y_F32 if f32_out else L.LUTGEMM_Y_F16
    torch.cuda.synchronize()
    L.lutgemm_gemv_static(d_x, p.d_bits, p.d_alpha, p.d_z, d_y, p.q, p.g, 8, p.m, p.n, flags,
                          torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return d_y.cpu().numpy()


def test_two_calls_in_a_row_second_one_smaller():
    cases = [(4100, 3072, 3, 128, L.LUTGEMM_Q_GREEDY), (515, 2048, 2, 64, L.LUTGEMM_Q_UNIFORM_RTN)]
    packed = []
    for (m, n, q, g, mode) in cases:
        W = synth.weights_fp16(m, n, seed=13000 + m)
        packed.append((Packed.from_weights(W, q, g, mode), synth.activations_fp16(n, seed=13500 + m)))
    got = [(_static(p, x, True), _static(p, x, False)) for p, x in packed]       # the two calls, back to back
    for (p, x), (y32, y16) in zip(packed, got):
        print(f"case static m={p.m} n={p.n} q={p.q} g={p.g}", flush=True)
        np.testing.assert_array_equal(y32, run(p, x, f32_out=True))
        np.testing.assert_array_equal(y16, run(p, x))
        gc = p.g
        a = O.decode_alpha(p.alpha, p.m, p.n // gc, p.q)
        z = None if p.z is None else O.decode_z(p.z, p.m, p.n // gc)
        y_ref = O.gemv_packed(p.bits, p.alpha, p.z, x, p.m, p.n, p.q, p.g)
        check_parity(y32, y_ref, x, row_l1_bound(a, z, gc), f32_out=True)
    # and once more on the first layer: the array is left ready by every call
    p, x = packed[0]
    np.testing.assert_array_equal(_static(p, x, True), got[0][0])


def test_layer_beyond_the_array_is_refused():
    torch = torch_cuda()
    m, n, q, g = 16, 8, 1, 8
    assert L.lutgemm_workspace_bytes(1 << 22, 8192, 3, 128) > L.lutgemm_static_scratch_bytes()
    d = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LutGemmError) as e:   # sizes are checked before any pointer is used
        L.lutgemm_gemv_static(d, d, d, None, d, 3, 128, 8, 1 << 22, 8192, 0, 0)
    assert e.value.code == L.LUTGEMM_EWORKSPACE
