"""CPU oracle for the BCQ / LUT-GEMM hot path (numpy, fp64).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; it is
used by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg.  It shares
no code, tables or helpers with the HIP library: the packed layouts are decoded here by
a decoder written from the layout text in include/lutgemm.h.

What each function follows
  dequant, gemv          the definition the method reaches exactly: section 3.3 eq. 3
                         (group-wise scales, section 3.4) then y = What x (section 3.2)
  lut_gemv               the method's own steps in the paper's order (section 3.1): tables
                         of 2^mu signed sums per sub-vector, keys from mu weight bits,
                         partial sums added, then scaled; counts the operations of eq. 2
  uniform_to_bcq         appendix C
  footprint_bits         section 3.4 eq. 4
  quantize_greedy,
  quantize_uniform_rtn   the quantiser arithmetic stated for the pack entry point in
                         include/lutgemm.h (the paper names no greedy quantiser)
  encode_* / decode_*    the packed layouts of include/lutgemm.h

Pins: tests/test_oracle_*.py (brute force over all 2^mu sign patterns, the sum(+-x)
identity, dense sum-of-planes + numpy.dot, linearity and negation, table identities,
the eq. 1 worked pattern, eq. 2 / eq. 4 / table 5 arithmetic, appendix C closed form,
hand-written packed bytes).  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

MU = 8


# ----------------------------------------------------------------------------------
# Definition: eq. 3 + matvec, all in fp64
# ----------------------------------------------------------------------------------
def dequant(B, alpha, z, g):
    """What[r][k] = sum_i alpha[i][r][k//g] * B[i][r][k] + z[r][k//g]   (section 3.3 eq. 3).

    B: int8 [q][m][n] in {-1,+1}; alpha: [q][m][n//g]; z: [m][n//g] or None.  fp64 out.
    """
    B = np.asarray(B)
    q, m, n = B.shape
    alpha = np.asarray(alpha, dtype=np.float64)
    assert n % g == 0 and alpha.shape == (q, m, n // g)
    What = np.zeros((m, n), dtype=np.float64)
    for i in range(q):
        What += np.repeat(alpha[i], g, axis=1) * B[i].astype(np.float64)
    if z is not None:
        z = np.asarray(z, dtype=np.float64)
        assert z.shape == (m, n // g)
        What += np.repeat(z, g, axis=1)
    return What


def gemv(B, alpha, z, g, x):
    """y[b][r] = sum_k What[r][k] x[b][k] in fp64 (section 3.2).  x: [n] or [batch][n]."""
    What = dequant(B, alpha, z, g)
    x = np.asarray(x, dtype=np.float64)
    if x.ndim == 1:
        return What @ x
    return (What @ x.T).T


# ----------------------------------------------------------------------------------
# The method itself, step by step (section 3.1), general mu
# ----------------------------------------------------------------------------------
def build_lut(xsub):
    """All 2^mu signed sums of one sub-vector: entry `key` adds x_j where bit j of key is
    1 and subtracts it where the bit is 0 (section 3.1)."""
    mu = len(xsub)
    lut = np.zeros(1 << mu, dtype=np.float64)
    for key in range(1 << mu):
        s = 0.0
        for j in range(mu):
            s += float(xsub[j]) if (key >> j) & 1 else -float(xsub[j])
        lut[key] = s
    return lut


def keys_of(Bplane, mu):
    """Keys of one plane: [m][n//mu] integers, bit j set iff the element is +1."""
    m, n = Bplane.shape
    assert n % mu == 0
    bits = (np.asarray(Bplane) > 0).astype(np.int64).reshape(m, n // mu, mu)
    return (bits << np.arange(mu, dtype=np.int64)).sum(axis=2)


def lut_gemv(B, alpha, z, g, x, mu=MU):
    """y = What x computed by table lookup, in the order section 3.1 gives: build the
    tables, look up every key, add the partial sums of a group, multiply by its scale.
    Returns (y, counts) with counts = {"build": table entries built, "read": lookups}
    (the two terms of eq. 2)."""
    B = np.asarray(B)
    q, m, n = B.shape
    assert n % mu == 0 and g % mu == 0 and n % g == 0
    x = np.asarray(x, dtype=np.float64)
    nsub = n // mu
    luts = [build_lut(x[c * mu:(c + 1) * mu]) for c in range(nsub)]
    counts = {"build": nsub * (1 << mu), "read": 0}
    y = np.zeros(m, dtype=np.float64)
    per_group = g // mu
    for i in range(q):
        keys = keys_of(B[i], mu)
        for r in range(m):
            for G in range(n // g):
                part = 0.0
                for c in range(G * per_group, (G + 1) * per_group):
                    part += luts[c][keys[r, c]]
                    counts["read"] += 1
                y[r] += float(alpha[i][r][G]) * part
    if z is not None:
        for r in range(m):
            for G in range(n // g):
                y[r] += float(z[r][G]) * float(x[G * g:(G + 1) * g].sum())
    return y, counts


# ----------------------------------------------------------------------------------
# Appendix C and eq. 4
# ----------------------------------------------------------------------------------
def uniform_to_bcq(u, s, zhat, q):
    """Appendix C: integer code u in [0, 2^q) with scale s and zero zhat, i.e.
    w = s*u + zhat, as BCQ: plane i is bit i of u mapped {0,1}->{-1,+1},
    alpha_i = 2^(i-1) s, z = zhat + sum_i alpha_i.  Returns (b[q] of +-1, alpha[q], z) fp64."""
    b = np.array([2 * ((int(u) >> i) & 1) - 1 for i in range(q)], dtype=np.float64)
    alpha = np.array([2.0 ** (i - 1) * float(s) for i in range(q)], dtype=np.float64)
    return b, alpha, float(zhat) + alpha.sum()


def footprint_bits(m, n, q, g, scale_bits=16):
    """Section 3.4 eq. 4: S = m n q (1 + scale_bits / g) bits."""
    return m * n * q + scale_bits * m * (n // g) * q


# ----------------------------------------------------------------------------------
# Quantisers (arithmetic fixed in include/lutgemm.h)
# ----------------------------------------------------------------------------------
def _seq_sum64(a):
    """fp64 sum along the last axis, strictly in increasing index order."""
    return np.add.accumulate(np.asarray(a, dtype=np.float64), axis=-1)[..., -1]


def quantize_greedy(W16, q, g, mean_offset=False):
    """Greedy BCQ of an fp16 matrix.  Returns (B int8 [q][m][n], alpha fp16 [q][m][NG],
    z fp16 [m][NG] or None)."""
    W16 = np.asarray(W16, dtype=np.float16)
    m, n = W16.shape
    g = n if g == 0 else g
    NG = n // g
    r = W16.astype(np.float32).reshape(m, NG, g)
    z = None
    if mean_offset:
        z = (_seq_sum64(r) / np.float64(g)).astype(np.float16)
        r = r - z.astype(np.float32)[:, :, None]
    B = np.empty((q, m, n), dtype=np.int8)
    alpha = np.empty((q, m, NG), dtype=np.float16)
    for i in range(q):
        b = np.where(r >= 0, np.float32(1), np.float32(-1))
        a = (_seq_sum64(np.abs(r)) / np.float64(g)).astype(np.float16)
        B[i] = b.reshape(m, n).astype(np.int8)
        alpha[i] = a
        r = (r - a.astype(np.float32)[:, :, None] * b).astype(np.float32)
    return B, alpha, z


def _solve_in_order(G, c):
    """Solve G a = c (q x q, fp64) by Gaussian elimination with partial pivoting, every
    operation in a fixed order (the packer does the same arithmetic).  None if singular."""
    q = len(c)
    A = [[float(G[i][j]) for j in range(q)] + [float(c[i])] for i in range(q)]
    for col in range(q):
        piv = col
        for r in range(col + 1, q):
            if abs(A[r][col]) > abs(A[piv][col]):
                piv = r
        if abs(A[piv][col]) < 1e-9:
            return None
        A[col], A[piv] = A[piv], A[col]
        for r in range(col + 1, q):
            f = A[r][col] / A[col][col]
            for j in range(col, q + 1):
                A[r][j] = A[r][j] - f * A[col][j]
    a = [0.0] * q
    for i in range(q - 1, -1, -1):
        acc = A[i][q]
        for j in range(i + 1, q):
            acc = acc - A[i][j] * a[j]
        a[i] = acc / A[i][i]
    return a


def _assign_codes(w, a):
    """For every weight the sign pattern (code: bit i = plane i is +1) whose level
    sum_i +-a_i is nearest; ties go to the smallest code.  Levels are summed in plane order."""
    q = len(a)
    levels = []
    for code in range(1 << q):
        v = 0.0
        for i in range(q):
            v = v + (a[i] if (code >> i) & 1 else -a[i])
        levels.append(v)
    codes = np.zeros(len(w), dtype=np.int64)
    for k, wk in enumerate(w):
        best, best_d = 0, abs(wk - levels[0])
        for code in range(1, 1 << q):
            d = abs(wk - levels[code])
            if d < best_d:
                best, best_d = code, d
        codes[k] = best
    return codes


def quantize_alternating_group(w16, q, iters=15):
    """Alternating BCQ of one group (the iterative solver the paper's appendix on compression
    ratios cites for obtaining BCQ weights): start from the greedy solution in fp64; then
    repeat { scales = least-squares fit for the current signs; planes with a negative scale
    are negated; every weight takes the nearest of the 2^q levels } until the signs stop
    changing or `iters` rounds have run; finally round the scales to fp16 and assign the
    signs once more for the stored scales.  Returns (b int8 [q][g], alpha fp16 [q])."""
    w = [float(v) for v in np.asarray(w16, dtype=np.float16).astype(np.float64)]
    g = len(w)
    r = list(w)
    b = [[0] * g for _ in range(q)]
    a = [0.0] * q
    for i in range(q):                                   # greedy start, fp64, sums in index order
        s = 0.0
        for k in range(g):
            b[i][k] = 1 if r[k] >= 0 else -1
            s = s + abs(r[k])
        a[i] = s / g
        for k in range(g):
            r[k] = r[k] - a[i] * b[i][k]
    for _ in range(iters):
        G = [[0.0] * q for _ in range(q)]
        c = [0.0] * q
        for i in range(q):
            for j in range(q):
                t = 0
                for k in range(g):
                    t += b[i][k] * b[j][k]
                G[i][j] = float(t)
            t = 0.0
            for k in range(g):
                t = t + b[i][k] * w[k]
            c[i] = t
        sol = _solve_in_order(G, c)
        if sol is None:                                  # two planes coincide: keep what we have
            break
        a = sol
        for i in range(q):
            if a[i] < 0:
                a[i] = -a[i]
                b[i] = [-v for v in b[i]]
        codes = _assign_codes(w, a)
        nb = [[1 if (int(codes[k]) >> i) & 1 else -1 for k in range(g)] for i in range(q)]
        if nb == b:
            break
        b = nb
    a16 = np.array(a, dtype=np.float64).astype(np.float16)
    codes = _assign_codes(w, [float(v) for v in a16.astype(np.float64)])
    B = np.array([[1 if (int(codes[k]) >> i) & 1 else -1 for k in range(g)] for i in range(q)], dtype=np.int8)
    return B, a16


def quantize_alternating(W16, q, g, iters=15):
    """Alternating BCQ of an fp16 matrix, group by group.  Returns (B int8 [q][m][n],
    alpha fp16 [q][m][NG], None)."""
    W16 = np.asarray(W16, dtype=np.float16)
    m, n = W16.shape
    g = n if g == 0 else g
    NG = n // g
    B = np.empty((q, m, n), dtype=np.int8)
    alpha = np.empty((q, m, NG), dtype=np.float16)
    for r in range(m):
        for G in range(NG):
            b, a = quantize_alternating_group(W16[r, G * g:(G + 1) * g], q, iters)
            B[:, r, G * g:(G + 1) * g] = b
            alpha[:, r, G] = a
    return B, alpha, None


def quantize_uniform_rtn(W16, q, g):
    """Asymmetric min/max round-to-nearest, converted to BCQ as appendix C states."""
    W16 = np.asarray(W16, dtype=np.float16)
    m, n = W16.shape
    g = n if g == 0 else g
    NG = n // g
    w = W16.astype(np.float32).reshape(m, NG, g)
    lo = w.min(axis=2)
    hi = w.max(axis=2)
    levels = np.float32((1 << q) - 1)
    with np.errstate(over="ignore"):
        s16 = ((hi - lo) / levels).astype(np.float32).astype(np.float16)
    s = s16.astype(np.float32)
    B = np.empty((q, m, n), dtype=np.int8)
    alpha = np.empty((q, m, NG), dtype=np.float16)
    with np.errstate(divide="ignore", invalid="ignore"):
        u = np.rint(((w - lo[:, :, None]) / s[:, :, None]).astype(np.float32))
    u = np.clip(u, 0, levels)
    u = np.where(s[:, :, None] == 0, levels, u).astype(np.int64)
    zsum = np.zeros((m, NG), dtype=np.float32)
    for i in range(q):
        a16 = (np.float32(2.0 ** (i - 1)) * s).astype(np.float32).astype(np.float16)
        alpha[i] = a16
        zsum = (zsum + a16.astype(np.float32)).astype(np.float32)
        B[i] = (2 * ((u >> i) & 1) - 1).reshape(m, n).astype(np.int8)
    z = (zsum + lo).astype(np.float32).astype(np.float16)
    return B, alpha, z


# ----------------------------------------------------------------------------------
# Packed layouts (written from the layout text of include/lutgemm.h)
# ----------------------------------------------------------------------------------
def _tiles(n):
    nchunks = n // 8
    NT = -(-nchunks // 128)
    out = []
    for kt in range(NT):
        C = min(128, nchunks - 128 * kt)
        out.append((kt, C, 2 if C > 64 else 1))
    return out


def bits_nbytes(m, n, q):
    RB = -(-m // 16)
    tiles = _tiles(n)
    return RB * q * 1024 * (2 * (len(tiles) - 1) + tiles[-1][2])


def _bit_offset(m, n, q, i, r, c):
    """Byte offset of key (plane i, row r, chunk c)."""
    RB = -(-m // 16)
    rb, rho = divmod(r, 16)
    kt = c // 128
    C = min(128, n // 8 - 128 * kt)
    T = 2 if C > 64 else 1
    L, t = divmod(c - 128 * kt, T)
    j, cq = divmod(L, 4)           # quad and slot within the quad
    k = rho // 4                   # the lane of the quad that owns this row
    slab = kt * RB * q * 2048 + ((rb * q + i) * T + t) * 1024
    return slab + (4 * j + k) * 16 + 4 * ((cq - k) % 4) + rho % 4


def encode_bits(B):
    """B int8 [q][m][n] -> packed bytes (uint8 array), plain loops over keys."""
    B = np.asarray(B)
    q, m, n = B.shape
    out = np.zeros(bits_nbytes(m, n, q), dtype=np.uint8)
    for i in range(q):
        keys = keys_of(B[i], 8)
        for r in range(m):
            for c in range(n // 8):
                out[_bit_offset(m, n, q, i, r, c)] = keys[r, c]
    return out


def decode_bits(packed, m, n, q):
    """packed bytes -> B int8 [q][m][n] in {-1,+1}.  Vectorised over (row, chunk) so the
    large shapes decode in seconds; the offsets are those of _bit_offset."""
    packed = np.asarray(packed, dtype=np.uint8).ravel()
    assert packed.size == bits_nbytes(m, n, q)
    RB = -(-m // 16)
    r = np.arange(m, dtype=np.int64)[:, None]
    c = np.arange(n // 8, dtype=np.int64)[None, :]
    rb, rho = r // 16, r % 16
    kt = c // 128
    C = np.minimum(128, n // 8 - 128 * kt)
    T = np.where(C > 64, 2, 1)
    L = (c - 128 * kt) // T
    t = (c - 128 * kt) % T
    j, cq, k = L // 4, L % 4, rho // 4
    B = np.empty((q, m, n), dtype=np.int8)
    for i in range(q):
        off = (kt * RB * q * 2048 + ((rb * q + i) * T + t) * 1024
               + (4 * j + k) * 16 + 4 * ((cq - k) % 4) + rho % 4)
        keys = packed[off]  # [m][n//8]
        bits = (keys[:, :, None] >> np.arange(8, dtype=np.uint8)) & 1
        B[i] = (2 * bits.astype(np.int8) - 1).reshape(m, n)
    return B


def encode_alpha(alpha):
    """alpha fp16 [q][m][NG] -> packed fp16 array of RB*NG*q*16 entries."""
    alpha = np.asarray(alpha, dtype=np.float16)
    q, m, NG = alpha.shape
    RB = -(-m // 16)
    out = np.zeros(RB * NG * q * 16, dtype=np.float16)
    for i in range(q):
        for r in range(m):
            for G in range(NG):
                out[((((r // 16) * NG + G) * 4 + (r % 16) // 4) * q + i) * 4 + r % 4] = alpha[i, r, G]
    return out


def decode_alpha(packed, m, NG, q):
    packed = np.asarray(packed).view(np.float16).ravel()
    RB = -(-m // 16)
    assert packed.size == RB * NG * q * 16
    a = packed.reshape(RB, NG, 4, q, 4)          # [rb][G][rho / 4][i][rho % 4]
    return np.ascontiguousarray(a.transpose(3, 0, 2, 4, 1).reshape(q, RB * 16, NG)[:, :m, :])


def encode_z(z):
    z = np.asarray(z, dtype=np.float16)
    m, NG = z.shape
    RB = -(-m // 16)
    out = np.zeros(RB * NG * 16, dtype=np.float16)
    for r in range(m):
        for G in range(NG):
            out[((r // 16) * NG + G) * 16 + r % 16] = z[r, G]
    return out


def decode_z(packed, m, NG):
    packed = np.asarray(packed).view(np.float16).ravel()
    RB = -(-m // 16)
    assert packed.size == RB * NG * 16
    a = packed.reshape(RB, NG, 16)               # [rb][G][rho]
    return np.ascontiguousarray(a.transpose(0, 2, 1).reshape(RB * 16, NG)[:m, :])


def share_scales(alpha):
    """Appendix C gives the planes of a uniformly quantised group the scales
    alpha_i = 2^i * alpha_0, so one stored value per (row, group) carries them all.
    alpha fp16-valued [q][m][NG] -> alpha_0 [m][NG]; raises if some alpha_i is not exactly
    2^i * alpha_0 (the scales of a greedy quantiser are not)."""
    a = np.asarray(alpha, dtype=np.float64)
    base = a[0]
    for i in range(a.shape[0]):
        if not np.array_equal(a[i], base * 2.0 ** i):
            raise ValueError("scales are not powers of two times the first plane's")
    return np.asarray(alpha)[0].astype(np.float16)


def expand_shared(alpha0, q):
    """alpha_0 [m][NG] -> alpha [q][m][NG] with alpha_i = 2^i * alpha_0 (fp64)."""
    a0 = np.asarray(alpha0, dtype=np.float64)
    return np.stack([a0 * 2.0 ** i for i in range(q)])


def encode_alpha_shared(alpha0):
    """Shared-scale layout: fp16 [row block][group][16 rows], the layout of the offsets."""
    return encode_z(alpha0)


def decode_alpha_shared(packed, m, NG):
    return decode_z(packed, m, NG)


def gemv_packed(bits, alpha_p, z_p, x, m, n, q, g, rows=None, alpha_shared=False):
    """y (fp64) straight from the packed buffers: decode, then the definition above.
    rows: optional 1-D index array; only those output rows are computed (the rest of the
    matrix is never dequantised), so single outputs of very large layers stay cheap."""
    g = n if g == 0 else g
    NG = n // g
    x = np.asarray(x, dtype=np.float64)
    if alpha_shared:   # one scale per (row, group); plane i has 2^i times it (appendix C)
        alpha = expand_shared(decode_alpha_shared(alpha_p, m, NG), q)
    else:
        alpha = decode_alpha(alpha_p, m, NG, q)
    z = None if z_p is None else decode_z(z_p, m, NG)
    if rows is None:
        B = decode_bits(bits, m, n, q)
        return gemv(B, alpha, z, g, x)
    rows = np.asarray(rows, dtype=np.int64)
    bits = np.asarray(bits, dtype=np.uint8).ravel()
    B = np.empty((q, rows.size, n), dtype=np.int8)
    for i in range(q):
        for a, r in enumerate(rows):
            for c in range(n // 8):
                key = int(bits[_bit_offset(m, n, q, i, int(r), c)])
                for j in range(8):
                    B[i, a, 8 * c + j] = 1 if (key >> j) & 1 else -1
    return gemv(B, alpha[:, rows, :], None if z is None else z[rows, :], g, x)
