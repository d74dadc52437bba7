"""Helpers of the GPU parity tests: upload packed buffers with torch (device memory and
streams only), call the C ABI through the ctypes binding, compare with the oracle."""
import numpy as np

import paper_2206_09557_amd as L


def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


class Packed:
    """Packed host buffers of one layer plus their device copies."""

    def __init__(self, bits, alpha, z, m, n, q, g):
        torch = torch_cuda()
        self.m, self.n, self.q, self.g = m, n, q, g
        self.bits, self.alpha, self.z = bits, alpha, z
        self.d_bits = torch.from_numpy(bits).cuda()
        self.d_alpha = torch.from_numpy(alpha.view(np.int16)).cuda()
        self.d_z = None if z is None else torch.from_numpy(z.view(np.int16)).cuda()

    def share(self):
        """Also hold the scales in the shared-scale layout (uniformly quantised layers)."""
        torch = torch_cuda()
        self.alpha_shared = L.lutgemm_share_scales(self.alpha, self.m, self.n, self.q, self.g)
        self.d_alpha_shared = torch.from_numpy(self.alpha_shared.view(np.int16)).cuda()
        return self

    @classmethod
    def from_weights(cls, W, q, g, mode=L.LUTGEMM_Q_GREEDY):
        bits, alpha, z = L.lutgemm_pack_bcq(W, q, g, mode=mode)
        return cls(bits, alpha, z, W.shape[0], W.shape[1], q, g)


def make_workspace(nbytes, stream=None):
    """A workspace prepared as the header asks: garbage everywhere, then
    lutgemm_workspace_init (which only has to zero the arrival counters)."""
    torch = torch_cuda()
    d_ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    d_ws.fill_(0xFF)
    torch.cuda.synchronize()
    s = torch.cuda.current_stream() if stream is None else stream
    L.lutgemm_workspace_init(d_ws, nbytes, s.cuda_stream)
    s.synchronize()
    return d_ws


def run(packed, x16, f32_out=False, stream=None, workspace=None, mfma=False, shared=False, auto=False, dequant=False):
    """y (numpy) of lutgemm_gemv (1-D x) or lutgemm_gemm (2-D x; lutgemm_gemm_mfma if mfma) for the packed layer.
    y is pre-filled with NaN: it must be fully overwritten, never read."""
    torch = torch_cuda()
    p = packed
    x16 = np.ascontiguousarray(x16, dtype=np.float16)
    batch = 1 if x16.ndim == 1 else x16.shape[0]
    d_x = torch.from_numpy(x16.view(np.int16)).cuda()
    ydt = torch.float32 if f32_out else torch.float16
    d_y = torch.full((batch, p.m), float("nan"), dtype=ydt, device="cuda")
    wsb = L.lutgemm_workspace_bytes(p.m, p.n, p.q, p.g, 8, batch)
    d_ws = make_workspace(wsb, stream) if workspace is None else workspace
    assert d_ws.numel() >= wsb
    s = torch.cuda.current_stream() if stream is None else stream
    flags = L.LUTGEMM_Y_F32 if f32_out else L.LUTGEMM_Y_F16
    d_alpha = p.d_alpha
    if shared:   # scales in the shared-scale layout
        flags |= L.LUTGEMM_ALPHA_SHARED
        d_alpha = p.d_alpha_shared
    if auto:     # lutgemm_gemm picks the path
        flags |= L.LUTGEMM_PATH_AUTO
    torch.cuda.synchronize()
    if dequant:   # the dequantise-then-multiply comparison kernel
        L.lutgemm_gemm_dequant_mfma(d_x, p.d_bits, d_alpha, p.d_z, d_y, p.q, p.g, 8, p.m, p.n, batch, flags, d_ws,
                                    d_ws.numel(), s.cuda_stream)
    elif mfma:
        L.lutgemm_gemm_mfma(d_x, p.d_bits, d_alpha, p.d_z, d_y, p.q, p.g, 8, p.m, p.n, batch, flags, d_ws,
                            d_ws.numel(), s.cuda_stream)
    elif x16.ndim == 1 and not dequant:
        L.lutgemm_gemv(d_x, p.d_bits, d_alpha, p.d_z, d_y, p.q, p.g, 8, p.m, p.n, flags, d_ws, d_ws.numel(),
                       s.cuda_stream)
    else:
        L.lutgemm_gemm(d_x, p.d_bits, d_alpha, p.d_z, d_y, p.q, p.g, 8, p.m, p.n, batch, flags, d_ws,
                       d_ws.numel(), s.cuda_stream)
    s.synchronize()
    y = d_y.cpu().numpy()
    return y[0] if x16.ndim == 1 else y


class RowBounds:
    """Per-row error bounds of a layer: `l1` = sum_G g * (sum_i alpha[i][r][G] + |z[r][G]|), a
    bound on the L1 norm of the dequantised row (the reading of "sum of alpha" that fp16
    outputs can meet), and `strict` = max_G (sum_i alpha[i][r][G] + |z[r][G]|), the literal
    reading, which the fp32 outputs are held to.  Indexing selects rows."""

    def __init__(self, l1, strict):
        self.l1, self.strict = l1, strict

    def __getitem__(self, sel):
        return RowBounds(self.l1[sel], self.strict[sel])


def row_l1_bound(alpha, z, g_cols):
    """RowBounds from decoded scales alpha[q][m][NG] and offsets z[m][NG] (or None)."""
    s = np.abs(alpha.astype(np.float64)).sum(axis=0)
    if z is not None:
        s = s + np.abs(z.astype(np.float64))
    return RowBounds(g_cols * s.sum(axis=1), s.max(axis=1))


def check_parity(y_gpu, y_ref, x16, rowbound, f32_out=False, fp16_weights=False):
    """Tolerances of the workload statement: relative L2 <= 1e-3 and max abs <=
    1e-2 * |x|_inf * sum(alpha), the sum read per row as a bound on the row's L1 norm.
    fp32 output is held to relative L2 <= 1e-5 and, element by element, to the literal
    reading |y - y_ref| <= 1e-2 * |x|_inf * max_G sum_i alpha[i][r][G] (about 1e-3 on the
    benchmark layers, far below any row's magnitude: a lost or stale partial sum fails it).
    fp16_weights: the output of the dequantising comparison kernel, whose method rounds every
    rebuilt weight to fp16: held to the fp16-output tolerances whatever its output type."""
    f32_out = f32_out and not fp16_weights
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    assert np.all(np.isfinite(y_gpu))
    rel = np.linalg.norm(y_gpu - y_ref) / max(np.linalg.norm(y_ref), 1e-30)
    assert rel <= (1e-5 if f32_out else 1e-3), f"relative L2 error {rel}"
    xinf = float(np.abs(np.asarray(x16, dtype=np.float64)).max())
    err = np.abs(y_gpu - y_ref)
    bad = err > 1e-2 * xinf * rowbound.l1 + 1e-30
    assert not bad.any(), f"max-abs bound broken at rows {np.flatnonzero(bad)[:8]}"
    if f32_out:
        bad = err > 1e-2 * xinf * rowbound.strict + 1e-30
        assert not bad.any(), (f"strict per-element bound broken at rows {np.flatnonzero(bad)[:8]}: "
                               f"errors {err[bad][:4]}, bounds {(1e-2 * xinf * rowbound.strict)[bad][:4]}")
    return rel
