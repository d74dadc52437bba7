"""ctypes loader for oracle_gemv.c (the streaming fp64 oracle).  Test infrastructure only.

build() compiles oracle/oracle_gemv.c with gcc into oracle/liboracle_gemv.so; load()
returns the library, building it when no built copy exists.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_gemv.c")
_LIB = os.environ.get("ORACLE_GEMV_LIB") or os.path.join(_HERE, "liboracle_gemv.so")   # (override: sanitizer build)
_lib = None


def build():
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_gemv_packed.restype = ctypes.c_int
        lib.oracle_gemv_packed.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int]
        _lib = lib
    return _lib


def gemv_packed(bits, alpha_p, z_p, x16, m, n, q, g, rows=None, nthreads=0):
    """fp64 y[batch][nrows] (or [nrows] for 1-D x) from the packed host buffers.
    Returns (y, threads_used)."""
    lib = load()
    bits = np.ascontiguousarray(np.asarray(bits).view(np.uint8).ravel())
    alpha_p = np.ascontiguousarray(np.asarray(alpha_p).view(np.uint16).ravel())
    x16 = np.ascontiguousarray(np.asarray(x16, dtype=np.float16))
    batch = 1 if x16.ndim == 1 else x16.shape[0]
    zp = None
    if z_p is not None:
        z_p = np.ascontiguousarray(np.asarray(z_p).view(np.uint16).ravel())
        zp = z_p.ctypes.data
    if rows is None:
        nrows, rp = m, None
    else:
        rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        nrows, rp = rows.size, rows.ctypes.data
    y = np.empty((batch, nrows), dtype=np.float64)
    used = lib.oracle_gemv_packed(bits.ctypes.data, alpha_p.ctypes.data, zp,
                                  x16.view(np.uint16).ctypes.data, m, n, q, g, batch,
                                  rp, nrows, y.ctypes.data, nthreads)
    if used < 0:
        raise ValueError("oracle_gemv_packed rejected its arguments")
    return (y[0] if x16.ndim == 1 else y), used
