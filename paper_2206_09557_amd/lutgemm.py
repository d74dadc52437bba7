"""ctypes binding of liblutgemm.so: same names as include/lutgemm.h, argument marshalling
only.  Host entry points take and return numpy arrays; device entry points take anything
with a `.data_ptr()` (torch tensors on the GPU) or a raw integer address.  There is no
fallback: if the built library is absent, loading raises."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# LUTGEMM_LIB names another build of the library (the host-only sanitizer build of
# tests/run_host_sanitizers.sh); entry points that build lacks raise when called.
LIB_PATH = os.environ.get("LUTGEMM_LIB") or os.path.join(_PKG, "liblutgemm.so")

LUTGEMM_OK, LUTGEMM_EINVAL, LUTGEMM_EUNSUPPORTED, LUTGEMM_EWORKSPACE, LUTGEMM_EHIP = 0, -1, -2, -3, -4
LUTGEMM_Q_GREEDY, LUTGEMM_Q_GREEDY_MEAN_OFFSET, LUTGEMM_Q_UNIFORM_RTN, LUTGEMM_Q_ALTERNATING = 0, 1, 2, 3
LUTGEMM_Y_F16, LUTGEMM_Y_F32, LUTGEMM_ALPHA_SHARED, LUTGEMM_PATH_AUTO = 0, 1, 2, 4

_c = ctypes
_SIGNATURES = {
    "lutgemm_bits_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int64, _c.c_int]),
    "lutgemm_alpha_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int64, _c.c_int, _c.c_int]),
    "lutgemm_z_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int64, _c.c_int]),
    "lutgemm_alpha_shared_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int64, _c.c_int]),
    "lutgemm_share_scales": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int, _c.c_int, _c.c_void_p]),
    "lutgemm_workspace_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int64, _c.c_int, _c.c_int, _c.c_int, _c.c_int]),
    "lutgemm_pack_bcq": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                    _c.c_void_p, _c.c_void_p, _c.c_void_p]),
    "lutgemm_unpack_bcq": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int, _c.c_int, _c.c_void_p]),
    "lutgemm_pack_planes": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int, _c.c_int, _c.c_void_p]),
    "lutgemm_pack_scales": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int, _c.c_int,
                                       _c.c_void_p, _c.c_void_p]),
    "lutgemm_workspace_init": (_c.c_int, [_c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "lutgemm_gemv": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                _c.c_int, _c.c_int, _c.c_int, _c.c_int64, _c.c_int64, _c.c_uint,
                                _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "lutgemm_gemv_group": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                      _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_uint,
                                      _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "lutgemm_group_workspace_bytes": (_c.c_size_t, [_c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int]),
    "lutgemm_gemv_static": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                       _c.c_int, _c.c_int, _c.c_int, _c.c_int64, _c.c_int64, _c.c_uint, _c.c_void_p]),
    "lutgemm_static_scratch_bytes": (_c.c_size_t, []),
    "lutgemm_gemm": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                _c.c_int, _c.c_int, _c.c_int, _c.c_int64, _c.c_int64, _c.c_int, _c.c_uint,
                                _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "lutgemm_gemm_mfma": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                     _c.c_int, _c.c_int, _c.c_int, _c.c_int64, _c.c_int64, _c.c_int, _c.c_uint,
                                     _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "lutgemm_gemm_dequant_mfma": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                             _c.c_int, _c.c_int, _c.c_int, _c.c_int64, _c.c_int64, _c.c_int, _c.c_uint,
                                             _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "lutgemm_plan_grid": (_c.c_int, [_c.c_int64, _c.c_int64, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p]),
    "lutgemm_stream_read": (_c.c_int, [_c.c_void_p, _c.c_size_t, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "lutgemm_strerror": (_c.c_char_p, [_c.c_int]),
}
EXPORTS = tuple(_SIGNATURES)

_lib = None


class LutGemmError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {lib().lutgemm_strerror(code).decode()} ({code})")


def lib():
    """The loaded library.  Raises if liblutgemm.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2206_09557_amd.build`")
        # The device buffers come from PyTorch, whose wheel carries its own HIP runtime.
        # Load it first so that this library resolves libamdhip64 to that same copy: two
        # HIP runtimes in one process do not see each other's allocations or streams.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            if os.environ.get("LUTGEMM_LIB") and not hasattr(handle, name):
                continue   # a host-only build: calling a device entry point raises AttributeError
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(code, where):
    if code != LUTGEMM_OK:
        raise LutGemmError(code, where)


def _addr(obj):
    if obj is None:
        return None
    if isinstance(obj, int):
        return obj
    if hasattr(obj, "data_ptr"):
        return obj.data_ptr()
    if isinstance(obj, np.ndarray):
        return obj.ctypes.data
    raise TypeError(f"cannot take the address of {type(obj)}")


# ---- sizes -------------------------------------------------------------------------
def lutgemm_bits_bytes(m, n, q):
    return lib().lutgemm_bits_bytes(m, n, q)


def lutgemm_alpha_bytes(m, n, q, g):
    return lib().lutgemm_alpha_bytes(m, n, q, g)


def lutgemm_z_bytes(m, n, g):
    return lib().lutgemm_z_bytes(m, n, g)


def lutgemm_alpha_shared_bytes(m, n, g):
    return lib().lutgemm_alpha_shared_bytes(m, n, g)


def lutgemm_workspace_bytes(m, n, q, g, mu=8, batch=1):
    return lib().lutgemm_workspace_bytes(m, n, q, g, mu, batch)


# ---- host ----------------------------------------------------------------------------
def lutgemm_pack_bcq(W, q, g, mu=8, mode=LUTGEMM_Q_GREEDY):
    """W: numpy fp16 [m][n].  Returns (bits uint8[], alpha fp16[], z fp16[] or None)."""
    W = np.ascontiguousarray(W)
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 array")
    m, n = W.shape
    nb, na, nz = lutgemm_bits_bytes(m, n, q), lutgemm_alpha_bytes(m, n, q, g), lutgemm_z_bytes(m, n, g)
    if nb == 0 or na == 0:
        raise LutGemmError(LUTGEMM_EINVAL, "lutgemm_pack_bcq")
    bits = np.empty(nb, dtype=np.uint8)
    alpha = np.empty(na // 2, dtype=np.float16)
    z = np.empty(nz // 2, dtype=np.float16) if mode in (LUTGEMM_Q_GREEDY_MEAN_OFFSET, LUTGEMM_Q_UNIFORM_RTN) else None
    _check(lib().lutgemm_pack_bcq(W.ctypes.data, m, n, q, g, mu, mode, bits.ctypes.data, alpha.ctypes.data,
                                  _addr(z)), "lutgemm_pack_bcq")
    return bits, alpha, z


def lutgemm_unpack_bcq(bits, m, n, q, mu=8):
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    if bits.size != lutgemm_bits_bytes(m, n, q):
        raise LutGemmError(LUTGEMM_EINVAL, "lutgemm_unpack_bcq")
    B = np.empty((q, m, n), dtype=np.int8)
    _check(lib().lutgemm_unpack_bcq(bits.ctypes.data, m, n, q, mu, B.ctypes.data), "lutgemm_unpack_bcq")
    return B


def lutgemm_pack_planes(B, mu=8):
    B = np.ascontiguousarray(B, dtype=np.int8)
    q, m, n = B.shape
    nb = lutgemm_bits_bytes(m, n, q)
    if nb == 0:
        raise LutGemmError(LUTGEMM_EINVAL, "lutgemm_pack_planes")
    bits = np.empty(nb, dtype=np.uint8)
    _check(lib().lutgemm_pack_planes(B.ctypes.data, m, n, q, mu, bits.ctypes.data), "lutgemm_pack_planes")
    return bits


def lutgemm_pack_scales(alpha, z, n, g):
    """alpha fp16 [q][m][NG], z fp16 [m][NG] or None -> packed (alpha, z)."""
    alpha = np.ascontiguousarray(alpha, dtype=np.float16)
    q, m, _ = alpha.shape
    na, nz = lutgemm_alpha_bytes(m, n, q, g), lutgemm_z_bytes(m, n, g)
    if na == 0:
        raise LutGemmError(LUTGEMM_EINVAL, "lutgemm_pack_scales")
    ap = np.empty(na // 2, dtype=np.float16)
    zp = None
    if z is not None:
        z = np.ascontiguousarray(z, dtype=np.float16)
        zp = np.empty(nz // 2, dtype=np.float16)
    _check(lib().lutgemm_pack_scales(alpha.ctypes.data, _addr(z), m, n, q, g, ap.ctypes.data, _addr(zp)),
           "lutgemm_pack_scales")
    return ap, zp


def lutgemm_share_scales(alpha_packed, m, n, q, g):
    """Packed per-plane scales (numpy fp16) -> shared-scale layout (numpy fp16)."""
    alpha_packed = np.ascontiguousarray(alpha_packed, dtype=np.float16)
    ns = lutgemm_alpha_shared_bytes(m, n, g)
    if ns == 0 or alpha_packed.nbytes != lutgemm_alpha_bytes(m, n, q, g):
        raise LutGemmError(LUTGEMM_EINVAL, "lutgemm_share_scales")
    out = np.empty(ns // 2, dtype=np.float16)
    _check(lib().lutgemm_share_scales(alpha_packed.ctypes.data, m, n, q, g, out.ctypes.data), "lutgemm_share_scales")
    return out


def lutgemm_plan_grid(m, n, q, g, vectors=1, compute_units=0):
    """(K groups, tiles per K group, row ranges) of the lookup kernel for `vectors` per pass."""
    out = (ctypes.c_int * 3)()
    _check(lib().lutgemm_plan_grid(m, n, q, g, vectors, compute_units, ctypes.addressof(out)), "lutgemm_plan_grid")
    return int(out[0]), int(out[1]), int(out[2])


# ---- device --------------------------------------------------------------------------
def lutgemm_workspace_init(workspace, workspace_bytes, stream=0):
    _check(lib().lutgemm_workspace_init(_addr(workspace), workspace_bytes, stream or None), "lutgemm_workspace_init")


def lutgemm_gemv(x, bits, alpha, z, y, q, g, mu, m, n, flags, workspace, workspace_bytes, stream=0):
    _check(lib().lutgemm_gemv(_addr(x), _addr(bits), _addr(alpha), _addr(z), _addr(y), q, g, mu, m, n, flags,
                              _addr(workspace), workspace_bytes, stream or None), "lutgemm_gemv")


def _pointer_array(objs):
    return (ctypes.c_void_p * len(objs))(*[_addr(o) for o in objs])


def _int64_array(values):
    return (ctypes.c_int64 * len(values))(*[int(v) for v in values])


def lutgemm_group_workspace_bytes(m, n, q, g, mu=8):
    """m, n: sequences of the layers' shapes."""
    return lib().lutgemm_group_workspace_bytes(_int64_array(m), _int64_array(n), len(m), q, g, mu)


def lutgemm_gemv_group(x, bits, alpha, z, y, m, n, q, g, mu, flags, workspace, workspace_bytes, stream=0):
    """x, bits, alpha, y (and z, or None): sequences of device buffers, one per layer."""
    count = len(m)
    zs = None if z is None else _pointer_array(z)
    _check(lib().lutgemm_gemv_group(_pointer_array(x), _pointer_array(bits), _pointer_array(alpha), zs,
                                    _pointer_array(y), _int64_array(m), _int64_array(n), count, q, g, mu, flags,
                                    _addr(workspace), workspace_bytes, stream or None), "lutgemm_gemv_group")


def lutgemm_gemv_static(x, bits, alpha, z, y, q, g, mu, m, n, flags, stream=0):
    _check(lib().lutgemm_gemv_static(_addr(x), _addr(bits), _addr(alpha), _addr(z), _addr(y), q, g, mu, m, n, flags,
                                     stream or None), "lutgemm_gemv_static")


def lutgemm_static_scratch_bytes():
    return lib().lutgemm_static_scratch_bytes()


def lutgemm_gemm(x, bits, alpha, z, y, q, g, mu, m, n, batch, flags, workspace, workspace_bytes, stream=0):
    _check(lib().lutgemm_gemm(_addr(x), _addr(bits), _addr(alpha), _addr(z), _addr(y), q, g, mu, m, n, batch,
                              flags, _addr(workspace), workspace_bytes, stream or None), "lutgemm_gemm")


def lutgemm_stream_read(src, nbytes, sink, sink_bytes, stream=0):
    _check(lib().lutgemm_stream_read(_addr(src), nbytes, _addr(sink), sink_bytes, stream or None), "lutgemm_stream_read")


def lutgemm_gemm_mfma(x, bits, alpha, z, y, q, g, mu, m, n, batch, flags, workspace, workspace_bytes, stream=0):
    _check(lib().lutgemm_gemm_mfma(_addr(x), _addr(bits), _addr(alpha), _addr(z), _addr(y), q, g, mu, m, n, batch,
                                   flags, _addr(workspace), workspace_bytes, stream or None), "lutgemm_gemm_mfma")


def lutgemm_gemm_dequant_mfma(x, bits, alpha, z, y, q, g, mu, m, n, batch, flags, workspace, workspace_bytes, stream=0):
    _check(lib().lutgemm_gemm_dequant_mfma(_addr(x), _addr(bits), _addr(alpha), _addr(z), _addr(y), q, g, mu, m, n,
                                           batch, flags, _addr(workspace), workspace_bytes, stream or None),
           "lutgemm_gemm_dequant_mfma")
