"""Pins of the oracle's greedy quantiser: least-squares identities of mean|r| with
b = sign(r), exact reproduction of constant-magnitude groups, sign(0) = +1."""
import numpy as np
import pytest

from oracle import bcq_oracle as O


def _exact_greedy_step(r):
    """One greedy pass in exact (fp64) arithmetic, no fp16 rounding of alpha."""
    b = np.where(r >= 0, 1.0, -1.0)
    a = np.abs(r).mean(axis=-1, keepdims=True)
    return b, a, r - a * b


def test_greedy_identities_in_exact_arithmetic():
    # mean|r| is the least-squares scale for b = sign(r):  sum b r = g a  and
    # |r'|^2 = |r|^2 - g a^2.  These pin what the quantiser is supposed to compute.
    rng = np.random.default_rng(21)
    r = rng.standard_normal((5, 4, 32)) * 0.02
    for _ in range(3):
        b, a, r2 = _exact_greedy_step(r)
        np.testing.assert_allclose((b * r).sum(-1, keepdims=True), 32 * a, rtol=1e-12)
        np.testing.assert_allclose((r2 ** 2).sum(-1), (r ** 2).sum(-1) - 32 * a[..., 0] ** 2, rtol=1e-9, atol=1e-18)
        r = r2


@pytest.mark.parametrize("mean_offset", [False, True])
def test_quantizer_tracks_exact_greedy(mean_offset):
    rng = np.random.default_rng(22)
    m, n, q, g = 6, 256, 3, 64
    W = (rng.standard_normal((m, n)) * 0.02).astype(np.float16)
    B, alpha, z = O.quantize_greedy(W, q, g, mean_offset=mean_offset)
    r = W.astype(np.float64).reshape(m, n // g, g)
    if mean_offset:
        zz = r.mean(-1)
        np.testing.assert_allclose(z.astype(np.float64), zz, rtol=2.0 ** -11, atol=6e-8)
        r = r - z.astype(np.float64)[:, :, None]
    else:
        assert z is None
    for i in range(q):
        b, a, _ = _exact_greedy_step(r)
        np.testing.assert_array_equal(B[i].reshape(m, n // g, g), b.astype(np.int8))
        # stored alpha = fp16 rounding of the exact mean (fp32 residual error is far below)
        np.testing.assert_allclose(alpha[i].astype(np.float64), a[..., 0], rtol=2.0 ** -11 + 1e-5, atol=6e-8)
        assert np.all(alpha[i] >= 0)
        r = r - alpha[i].astype(np.float64)[:, :, None] * b      # the ROUNDED alpha is subtracted
    # reconstruction error after q passes equals the final residual
    What = O.dequant(B, alpha, z, g)
    np.testing.assert_allclose(W.astype(np.float64) - What, r.reshape(m, n), rtol=0, atol=1e-7)


def test_constant_magnitude_group_is_exact_and_sign_zero_is_plus():
    W = np.zeros((2, 32), dtype=np.float16)
    W[0, :16] = np.float16(0.375) * np.array([1, -1] * 8, dtype=np.float16)
    W[0, 16:] = 0.0                      # an all-zero group: alpha = 0, signs +1
    W[1, :16] = np.float16(-0.5)
    W[1, 16:] = np.float16(0.25) * np.array([1, 1, -1, -1] * 4, dtype=np.float16)
    B, alpha, z = O.quantize_greedy(W, 1, 16)
    np.testing.assert_array_equal(O.dequant(B, alpha, None, 16), W.astype(np.float64))
    assert np.all(B[0, 0, 16:] == 1) and alpha[0, 0, 1] == 0
    # second plane of an exactly represented group has zero residual: bits +1, alpha 0
    B2, alpha2, _ = O.quantize_greedy(W, 2, 16)
    assert np.all(B2[1] == 1) and np.all(alpha2[1] == 0)


def test_greedy_scales_need_not_decrease():
    # |r| = {0,0,0,4}: alpha0 = 1, then |r'| = {1,1,1,3}: alpha1 = 1.5 > alpha0
    W = np.array([[0, 0, 0, 4, 0, 0, 0, 4]], dtype=np.float16)
    _, alpha, _ = O.quantize_greedy(W, 2, 8)
    assert float(alpha[0, 0, 0]) == 1.0 and float(alpha[1, 0, 0]) == 1.5


def test_rowwise_group_zero_means_whole_row():
    rng = np.random.default_rng(23)
    W = (rng.standard_normal((3, 64)) * 0.02).astype(np.float16)
    B0, a0, _ = O.quantize_greedy(W, 2, 0)
    B1, a1, _ = O.quantize_greedy(W, 2, 64)
    np.testing.assert_array_equal(B0, B1)
    np.testing.assert_array_equal(a0, a1)


# ---- alternating BCQ (the iterative solver cited for obtaining BCQ weights) ----

def _sq_err(w16, B, alpha16):
    w = np.asarray(w16, dtype=np.float16).astype(np.float64)
    a = np.asarray(alpha16).astype(np.float64)
    return float(((w - (a[:, None] * B).sum(axis=0)) ** 2).sum())


def test_alternating_one_plane_is_the_closed_form():
    # q = 1: the least-squares scale for b = sign(w) is mean|w|, and sign(w) is the nearest level
    rng = np.random.default_rng(40)
    w = (rng.standard_normal(64) * 0.02).astype(np.float16)
    B, a = O.quantize_alternating_group(w, 1)
    np.testing.assert_array_equal(B[0], np.where(w.astype(np.float64) >= 0, 1, -1))
    assert a[0] == np.float16(np.abs(w.astype(np.float64)).mean())


def test_alternating_is_no_worse_than_greedy_and_a_fixed_point():
    rng = np.random.default_rng(41)
    worse = 0
    for trial in range(30):
        q = int(rng.integers(2, 5))
        g = int(rng.choice([8, 16, 64]))
        w = (rng.standard_normal(g) * 0.02).astype(np.float16)
        B, a = O.quantize_alternating_group(w, q)
        Bg, ag, _ = O.quantize_greedy(w[None, :], q, g)
        e_alt, e_greedy = _sq_err(w, B, a), _sq_err(w, Bg[:, 0, :], ag[:, 0, 0])
        assert e_alt <= e_greedy * (1 + 1e-3) + 1e-12
        worse += e_alt > e_greedy
        assert np.all(a.astype(np.float64) >= 0)
        # the signs are the nearest levels for the stored scales (second half-step is a fixed point)
        codes = O._assign_codes(w.astype(np.float64), [float(v) for v in a.astype(np.float64)])
        for i in range(q):
            np.testing.assert_array_equal(B[i], np.where((codes >> i) & 1, 1, -1))
    assert worse <= 2          # fp16 rounding of the scales can cost a hair, the iteration cannot


def test_alternating_against_brute_force_on_a_tiny_group():
    # g = 6, q = 2: all 2^12 sign matrices, least-squares scales for each (numpy lstsq);
    # the alternating result is a local optimum: never below the global one, on these seeds
    # equal to it four times out of five and within a factor of two otherwise; the greedy
    # start is at least as far
    rng = np.random.default_rng(42)
    for trial in range(5):
        w = (rng.standard_normal(6) * 0.02).astype(np.float16)
        w64 = w.astype(np.float64)
        best = np.inf
        for code in range(1 << 12):
            Bm = np.array([[1.0 if (code >> (i * 6 + k)) & 1 else -1.0 for k in range(6)] for i in range(2)])
            sol, *_ = np.linalg.lstsq(Bm.T, w64, rcond=None)
            best = min(best, float(((w64 - Bm.T @ sol) ** 2).sum()))
        B, a = O.quantize_alternating_group(w, 2)
        e_alt = _sq_err(w, B, a)
        ulp_slack = 6 * (2.0 ** -11 * np.abs(w64).max()) ** 2 * 4     # fp16 rounding of two scales
        assert e_alt >= best - 1e-15
        assert e_alt <= best * 2.0 + ulp_slack
        Bg, ag, _ = O.quantize_greedy(w[None, :], 2, 6)
        assert _sq_err(w, Bg[:, 0, :], ag[:, 0, 0]) >= e_alt - ulp_slack


def test_alternating_reproduces_exact_bcq_weights():
    # weights that ARE a 2-plane BCQ combination with dyadic scales are recovered exactly
    rng = np.random.default_rng(43)
    b = rng.choice([-1, 1], size=(2, 32))
    w = (0.5 * b[0] + 0.125 * b[1]).astype(np.float16)
    B, a = O.quantize_alternating_group(w, 2)
    np.testing.assert_array_equal((a.astype(np.float64)[:, None] * B).sum(axis=0), w.astype(np.float64))


def test_solver_against_numpy_and_singular_case():
    rng = np.random.default_rng(44)
    for q in (1, 2, 3, 5, 8):
        Bm = rng.choice([-1.0, 1.0], size=(q, 64))
        G = Bm @ Bm.T
        c = Bm @ rng.standard_normal(64)
        np.testing.assert_allclose(O._solve_in_order(G.tolist(), c.tolist()), np.linalg.solve(G, c), rtol=1e-10, atol=1e-12)
    assert O._solve_in_order([[4.0, -4.0], [-4.0, 4.0]], [1.0, -1.0]) is None
