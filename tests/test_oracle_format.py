"""Pins of the oracle's table semantics, operation counts, footprint arithmetic, the
appendix C conversion and the packed layouts (hand-written bytes)."""
import os

import numpy as np
import pytest

from oracle import bcq_oracle as O


# ---- table semantics (section 3.1) ---------------------------------------------------
def test_lut_identities():
    rng = np.random.default_rng(11)
    x = rng.standard_normal(8).astype(np.float16).astype(np.float64)
    lut = O.build_lut(x)
    assert lut.shape == (256,)
    for k in range(256):
        assert abs(lut[k] + lut[k ^ 0xFF]) < 1e-13            # complement negates
        for j in range(8):
            d = lut[k ^ (1 << j)] - lut[k]
            want = -2 * x[j] if (k >> j) & 1 else 2 * x[j]    # flipping one sign moves by 2 x_j
            assert abs(d - want) < 1e-12
    assert abs(lut[0xFF] - x.sum()) < 1e-13
    assert abs(lut[0] + x.sum()) < 1e-13


def test_eq1_key_sharing(golden_dir):
    # Section 3.1 eq. 1 with mu = 3: (x1 + x2 - x3) occurs three times, (-x4 - x5 + x6) twice.
    rows = [l.split() for l in open(os.path.join(golden_dir, "eq1_binary_matrix.txt"))
            if l.strip() and not l.startswith("#")]
    B = np.array([[int(v) for v in r] for r in rows], dtype=np.int8)
    assert B.shape == (4, 6)
    keys = O.keys_of(B, 3)
    first, second = keys[:, 0].tolist(), keys[:, 1].tolist()
    key_ppm = 0b011     # bits 0,1 set: +x1 +x2 -x3
    key_mmp = 0b100     # bit 2 set:    -x4 -x5 +x6
    assert first.count(key_ppm) == 3 and second.count(key_mmp) == 2
    assert len(set(first)) == 2 and len(set(second)) == 3
    # and the lookup result equals the plain product for a random x
    x = np.random.default_rng(12).standard_normal(6)
    y, counts = O.lut_gemv(B[None], np.ones((1, 4, 2)), None, 3, x, mu=3)
    np.testing.assert_allclose(y, B.astype(np.float64) @ x, atol=1e-13)
    assert counts == {"build": 2 * 8, "read": 4 * 2}


@pytest.mark.parametrize("m,n,q,g,mu", [(6, 64, 3, 16, 8), (9, 48, 2, 24, 4), (4, 64, 1, 64, 8)])
def test_lut_method_equals_definition_and_eq2_counts(m, n, q, g, mu):
    rng = np.random.default_rng(13)
    B = rng.choice(np.array([-1, 1], dtype=np.int8), size=(q, m, n))
    alpha = np.abs(rng.standard_normal((q, m, n // g))).astype(np.float16)
    z = rng.standard_normal((m, n // g)).astype(np.float16)
    x = rng.standard_normal(n).astype(np.float16)
    y, counts = O.lut_gemv(B, alpha, z, g, x, mu=mu)
    np.testing.assert_allclose(y, O.gemv(B, alpha, z, g, x), rtol=0, atol=1e-11)
    # eq. 2: C_build = 2^mu * n/mu entries, C_read = m * (n/mu) * q lookups
    assert counts["build"] == (1 << mu) * n // mu
    assert counts["read"] == m * (n // mu) * q


# ---- footprint (section 3.4 eq. 4, table 5) -----------------------------------------
def test_eq4_and_table5(golden_dir):
    m, n = 49152, 12288
    # eq. 4 as printed: bits + 16-bit scales, q per group
    assert O.footprint_bits(m, n, 3, 128) == m * n * 3 + 16 * m * (n // 128) * 3
    assert O.bits_nbytes(m, n, 3) * 8 == m * n * 3                   # binary term, exact
    rows = [l.split() for l in open(os.path.join(golden_dir, "table5_compression.txt"))
            if l.strip() and not l.startswith("#")]
    for qs, gs, ratio in rows:
        q, ratio = int(qs), float(ratio)
        if gs == "-":
            # row-wise: 16 / q up to the (negligible) scale term
            got = 16.0 * m * n / O.footprint_bits(m, n, q, n)
            assert abs(got - ratio) < 0.01
            assert abs(16.0 / q - ratio) < 0.006
        else:
            # the printed group-wise ratios correspond to ONE 16-bit value per group,
            # 16 / (q + 16/g); eq. 4's q scales per group gives a smaller ratio.
            g = int(gs)
            assert abs(16.0 / (q + 16.0 / g) - ratio) < 0.006
            assert 16.0 * m * n / O.footprint_bits(m, n, q, g) < ratio


# ---- appendix C ------------------------------------------------------------------------
@pytest.mark.parametrize("q", [1, 2, 3, 4, 8])
def test_uniform_to_bcq_closed_form(q):
    s, zhat = 0.1875, -1.25          # dyadic: every product and sum below is exact
    for u in range(1 << q):
        b, alpha, z = O.uniform_to_bcq(u, s, zhat, q)
        assert set(np.abs(b)) == {1.0}
        assert float(alpha @ b + z) == s * u + zhat
        assert alpha[0] == s / 2 and all(alpha[i] == 2 * alpha[i - 1] for i in range(1, q))


def test_uniform_rtn_quantizer_reproduces_grid_points():
    # weights that already sit on a uniform grid are reproduced exactly by the
    # uniform -> BCQ route (dyadic step and zero so that fp16 holds everything exactly)
    q, g = 3, 16
    s, zhat = 0.125, -0.5
    rng = np.random.default_rng(14)
    u = rng.integers(0, 1 << q, size=(7, 64))
    u[:, ::16] = 0
    u[:, 1::16] = (1 << q) - 1           # every group spans the whole range
    W = (s * u + zhat).astype(np.float16)
    B, alpha, z = O.quantize_uniform_rtn(W, q, g)
    np.testing.assert_array_equal(O.dequant(B, alpha, z, g), W.astype(np.float64))
    assert np.all(alpha[0] == np.float16(s / 2)) and np.all(z == np.float16(zhat + s * 3.5))
    # planes are the bits of u
    for i in range(q):
        np.testing.assert_array_equal(B[i], 2 * ((u >> i) & 1) - 1)


def test_uniform_rtn_error_bound_and_degenerate_group():
    rng = np.random.default_rng(15)
    W = (rng.standard_normal((9, 128)) * 0.02).astype(np.float16)
    W[3, 32:64] = np.float16(0.0123)     # constant group: s = 0
    q, g = 4, 32
    B, alpha, z = O.quantize_uniform_rtn(W, q, g)
    What = O.dequant(B, alpha, z, g)
    w = W.astype(np.float64).reshape(9, 4, 32)
    step = alpha[0].astype(np.float64) * 2            # [9][4]
    err = np.abs(What.reshape(9, 4, 32) - w)
    # half a step plus the fp16 roundings of s (range/(2^q-1)) and of z
    bound = 0.5 * step[:, :, None] + 15 * 2.0 ** -11 * step[:, :, None] + 2.0 ** -11 * np.abs(z.astype(np.float64))[:, :, None] + 1e-7
    assert np.all(err <= bound)
    assert np.all(B[:, 3, 32:64] == 1) and np.all(alpha[:, 3, 1] == 0) and z[3, 1] == np.float16(0.0123)


def test_shared_scales_are_the_appendix_c_scales():
    # appendix C: alpha_i = 2^i * alpha_0 for a uniformly quantised group, so alpha_0 alone
    # carries the scales; the shared form gives the same dequantised weights and products
    rng = np.random.default_rng(16)
    W = (rng.standard_normal((21, 256)) * 0.02).astype(np.float16)
    q, g = 4, 64
    B, alpha, z = O.quantize_uniform_rtn(W, q, g)
    a0 = O.share_scales(alpha)
    assert a0.dtype == np.float16 and a0.shape == (21, 4)
    np.testing.assert_array_equal(O.expand_shared(a0, q), alpha.astype(np.float64))
    for i in range(q):                                   # closed form of the conversion
        np.testing.assert_array_equal(alpha[i].astype(np.float64), a0.astype(np.float64) * 2.0 ** i)
    x = rng.standard_normal(256).astype(np.float16)
    bits = O.encode_bits(B)
    y_planes = O.gemv_packed(bits, O.encode_alpha(alpha), O.encode_z(z), x, 21, 256, q, g)
    y_shared = O.gemv_packed(bits, O.encode_alpha_shared(a0), O.encode_z(z), x, 21, 256, q, g, alpha_shared=True)
    np.testing.assert_array_equal(y_planes, y_shared)
    # and against the integer form  w = s * u + zhat  with s = 2 * alpha_0 (dense numpy product)
    u = sum(((B[i] + 1) // 2).astype(np.int64) << i for i in range(q))
    s_full = np.repeat(2.0 * a0.astype(np.float64), g, axis=1)
    zhat = np.repeat(z.astype(np.float64) - a0.astype(np.float64) * (2 ** q - 1), g, axis=1)
    np.testing.assert_allclose((s_full * u + zhat) @ x.astype(np.float64), y_shared, rtol=1e-12, atol=1e-12)
    # scales of a greedy quantiser are not of that form
    _, alpha_g, _ = O.quantize_greedy(W, 3, g)
    with pytest.raises(ValueError):
        O.share_scales(alpha_g)


# ---- packed layouts: hand-written bytes ------------------------------------------------
def _load_layout_cases(golden_dir):
    cases, cur, extra = [], None, []
    for line in open(os.path.join(golden_dir, "packed_layout.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "case":
            cur = {"m": int(t[1]), "n": int(t[2]), "q": int(t[3]), "plus": [], "allplus": [], "bytes": {}}
            cases.append(cur)
        elif t[0] == "plus":
            cur["plus"].append(tuple(int(v) for v in t[1:]))
        elif t[0] == "allplus":
            cur["allplus"].append(tuple(int(v) for v in t[1:]))
        elif t[0] == "size":
            cur["size"] = int(t[1])
        elif t[0] == "byte":
            cur["bytes"][int(t[1])] = int(t[2], 16)
        else:
            extra.append(t)
    return cases, extra


def layout_case_planes(case):
    B = -np.ones((case["q"], case["m"], case["n"]), dtype=np.int8)
    for i, r, k in case["plus"]:
        B[i, r, k] = 1
    for i, r in case["allplus"]:
        B[i, r, :] = 1
    return B


def test_packed_bits_match_hand_written_bytes(golden_dir):
    cases, _ = _load_layout_cases(golden_dir)
    assert len(cases) == 3
    for case in cases:
        B = layout_case_planes(case)
        packed = O.encode_bits(B)
        assert packed.size == case["size"] == O.bits_nbytes(case["m"], case["n"], case["q"])
        want = np.zeros(case["size"], dtype=np.uint8)
        for off, val in case["bytes"].items():
            want[off] = val
        np.testing.assert_array_equal(packed, want)
        np.testing.assert_array_equal(O.decode_bits(packed, case["m"], case["n"], case["q"]), B)


def test_packed_scale_indices_match_hand_written(golden_dir):
    _, extra = _load_layout_cases(golden_dir)
    seen = 0
    for t in extra:
        if t[0] == "alpha":
            m, NG, q, i, r, G, idx = (int(v) for v in t[1:])
            a = np.zeros((q, m, NG), dtype=np.float16)
            a[i, r, G] = 1.5
            p = O.encode_alpha(a)
            assert p.size == -(-m // 16) * NG * q * 16
            assert np.flatnonzero(p).tolist() == [idx]
            np.testing.assert_array_equal(O.decode_alpha(p, m, NG, q), a)
        elif t[0] == "z":
            m, NG, r, G, idx = (int(v) for v in t[1:])
            z = np.zeros((m, NG), dtype=np.float16)
            z[r, G] = -2.0
            p = O.encode_z(z)
            assert p.size == -(-m // 16) * NG * 16
            assert np.flatnonzero(p).tolist() == [idx]
            np.testing.assert_array_equal(O.decode_z(p, m, NG), z)
        elif t[0] == "shared":
            m, NG, r, G, idx = (int(v) for v in t[1:])
            a0 = np.zeros((m, NG), dtype=np.float16)
            a0[r, G] = 0.75
            p = O.encode_alpha_shared(a0)
            assert p.size == -(-m // 16) * NG * 16
            assert np.flatnonzero(p).tolist() == [idx]
            np.testing.assert_array_equal(O.decode_alpha_shared(p, m, NG), a0)
        seen += 1
    assert seen == 7


@pytest.mark.parametrize("m,n,q", [(1, 8, 1), (17, 520, 3), (33, 1544, 2), (16, 2048, 4), (50, 1024 + 512, 3)])
def test_bits_roundtrip_and_popcount(m, n, q):
    rng = np.random.default_rng(16)
    B = rng.choice(np.array([-1, 1], dtype=np.int8), size=(q, m, n))
    packed = O.encode_bits(B)
    np.testing.assert_array_equal(O.decode_bits(packed, m, n, q), B)
    pop = int(np.unpackbits(packed).sum())
    assert pop == int((B > 0).sum())                  # padding bytes are zero
