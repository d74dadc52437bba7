"""Pins of the oracle's matvec (numpy and C) against things fixed by the mathematics:
brute force over all 2^mu sign patterns, the sum(+-x) identity, a dense sum-of-planes
matrix handed to numpy.dot, linearity, negation, and planted-mistake detection."""
import itertools

import numpy as np
import pytest

from oracle import bcq_oracle as O
from oracle import c_oracle


def _rand_case(rng, m, n, q, g, with_z):
    B = rng.choice(np.array([-1, 1], dtype=np.int8), size=(q, m, n))
    alpha = np.abs(rng.standard_normal((q, m, n // g))).astype(np.float16)
    z = rng.standard_normal((m, n // g)).astype(np.float16) if with_z else None
    x = rng.standard_normal(n).astype(np.float16)
    return B, alpha, z, x


def _both(B, alpha, z, g, x):
    """y from the numpy definition and from the C oracle through the packed buffers."""
    q, m, n = B.shape
    y_np = O.gemv(B, alpha, z, g, x)
    bits = O.encode_bits(B)
    ap = O.encode_alpha(alpha)
    zp = None if z is None else O.encode_z(z)
    y_c, _ = c_oracle.gemv_packed(bits, ap, zp, x, m, n, q, g)
    y_np2 = O.gemv_packed(bits, ap, zp, x, m, n, q, g)
    return y_np, y_c, y_np2


def test_brute_force_all_sign_patterns():
    # n = mu = 8, one plane, one row per sign pattern: y_r is a literal signed sum.
    rng = np.random.default_rng(1)
    x = rng.standard_normal(8).astype(np.float16)
    a = np.float16(0.75)
    patterns = list(itertools.product([-1, 1], repeat=8))
    B = np.array(patterns, dtype=np.int8)[None]           # [1][256][8]
    alpha = np.full((1, 256, 1), a, dtype=np.float16)
    expect = np.empty(256)
    for r, pat in enumerate(patterns):
        s = 0.0
        for k in range(8):
            s += pat[k] * float(x[k])
        expect[r] = float(a) * s
    for y in _both(B, alpha, None, 8, x):
        np.testing.assert_allclose(y, expect, rtol=0, atol=1e-13)


def test_brute_force_two_planes_with_offset():
    # q = 2, n = 8, every pair of patterns from a reduced set, plus offset: literal loops.
    rng = np.random.default_rng(2)
    x = rng.standard_normal(8).astype(np.float16)
    pats = [p for p in itertools.product([-1, 1], repeat=8)][::17]
    rows = [(p0, p1) for p0 in pats for p1 in pats]
    m = len(rows)
    B = np.empty((2, m, 8), dtype=np.int8)
    alpha = np.abs(rng.standard_normal((2, m, 1))).astype(np.float16)
    z = rng.standard_normal((m, 1)).astype(np.float16)
    expect = np.empty(m)
    for r, (p0, p1) in enumerate(rows):
        B[0, r], B[1, r] = p0, p1
        s = 0.0
        for k in range(8):
            w = float(alpha[0, r, 0]) * p0[k] + float(alpha[1, r, 0]) * p1[k] + float(z[r, 0])
            s += w * float(x[k])
        expect[r] = s
    for y in _both(B, alpha, z, 8, x):
        np.testing.assert_allclose(y, expect, rtol=0, atol=1e-12)


@pytest.mark.parametrize("n", [8, 64, 1032])
def test_unit_scale_is_signed_sum(n):
    # q = 1, alpha = 1, z = 0  =>  y_r = sum_k +-x_k
    rng = np.random.default_rng(3)
    m = 19
    B = rng.choice(np.array([-1, 1], dtype=np.int8), size=(1, m, n))
    alpha = np.ones((1, m, 1), dtype=np.float16)
    x = rng.standard_normal(n).astype(np.float16)
    expect = np.array([sum(float(x[k]) if B[0, r, k] > 0 else -float(x[k]) for k in range(n))
                       for r in range(m)])
    for y in _both(B, alpha, None, n, x):
        np.testing.assert_allclose(y, expect, rtol=0, atol=1e-11)


@pytest.mark.parametrize("m,n,q,g,with_z", [(5, 64, 3, 16, False), (33, 1544, 2, 8, True),
                                             (16, 1536, 4, 128, True), (40, 2048, 3, 2048, False)])
def test_dense_sum_of_planes_numpy_dot(m, n, q, g, with_z):
    rng = np.random.default_rng(4)
    B, alpha, z, x = _rand_case(rng, m, n, q, g, with_z)
    dense = np.zeros((m, n))
    for i in range(q):
        for G in range(n // g):
            dense[:, G * g:(G + 1) * g] += alpha[i, :, G:G + 1].astype(np.float64) * B[i, :, G * g:(G + 1) * g]
    if with_z:
        for G in range(n // g):
            dense[:, G * g:(G + 1) * g] += z[:, G:G + 1].astype(np.float64)
    expect = np.dot(dense, x.astype(np.float64))
    for y in _both(B, alpha, z, g, x):
        np.testing.assert_allclose(y, expect, rtol=1e-12, atol=1e-11)


def test_linearity_and_negation():
    rng = np.random.default_rng(5)
    B, alpha, z, x1 = _rand_case(rng, 12, 256, 3, 32, True)
    x2 = rng.standard_normal(256).astype(np.float16).astype(np.float64)
    x1 = x1.astype(np.float64)
    y1, y2, y12 = O.gemv(B, alpha, z, 32, x1), O.gemv(B, alpha, z, 32, x2), O.gemv(B, alpha, z, 32, x1 + x2)
    np.testing.assert_allclose(y12, y1 + y2, rtol=0, atol=1e-11)
    # without offset, flipping every sign negates y
    ya = O.gemv(B, alpha, None, 32, x1)
    yb = O.gemv(-B, alpha, None, 32, x1)
    np.testing.assert_allclose(ya, -yb, rtol=0, atol=1e-12)


def test_batch_rows_are_independent_gemvs():
    rng = np.random.default_rng(6)
    B, alpha, z, _ = _rand_case(rng, 20, 128, 3, 64, True)
    X = rng.standard_normal((5, 128)).astype(np.float16)
    Y = O.gemv(B, alpha, z, 64, X)
    bits, ap, zp = O.encode_bits(B), O.encode_alpha(alpha), O.encode_z(z)
    Yc, _ = c_oracle.gemv_packed(bits, ap, zp, X, 20, 128, 3, 64)
    for b in range(5):
        yb = O.gemv(B, alpha, z, 64, X[b])
        np.testing.assert_allclose(Y[b], yb, rtol=0, atol=1e-12)
        np.testing.assert_allclose(Yc[b], yb, rtol=0, atol=1e-11)


def test_row_subset_matches_full():
    rng = np.random.default_rng(7)
    m, n, q, g = 50, 1544, 3, 8
    B, alpha, z, x = _rand_case(rng, m, n, q, g, True)
    bits, ap, zp = O.encode_bits(B), O.encode_alpha(alpha), O.encode_z(z)
    full = O.gemv(B, alpha, z, g, x)
    rows = np.array([49, 0, 16, 17, 33])
    sub_np = O.gemv_packed(bits, ap, zp, x, m, n, q, g, rows=rows)
    sub_c, _ = c_oracle.gemv_packed(bits, ap, zp, x, m, n, q, g, rows=rows)
    np.testing.assert_allclose(sub_np, full[rows], rtol=0, atol=1e-11)
    np.testing.assert_allclose(sub_c, full[rows], rtol=0, atol=1e-11)


def test_planted_mistakes_are_caught():
    # The pins above must be able to fail: a dropped plane, a transposed scale index, a
    # flipped polarity and a dropped offset each move y far beyond the pin tolerance.
    rng = np.random.default_rng(8)
    B, alpha, z, x = _rand_case(rng, 8, 64, 2, 16, True)
    good = O.gemv(B, alpha, z, 16, x)
    assert np.abs(O.gemv(B[:1], alpha[:1], z, 16, x) - good).max() > 1e-3
    assert np.abs(O.gemv(B, alpha[:, :, ::-1], z, 16, x) - good).max() > 1e-3
    assert np.abs(O.gemv(-B, alpha, z, 16, x) - good).max() > 1e-3
    assert np.abs(O.gemv(B, alpha, None, 16, x) - good).max() > 1e-3
