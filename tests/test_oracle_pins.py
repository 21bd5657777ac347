"""Pins for the CPU oracle: each test checks it against something fixed by the
paper or by mathematics, not against its own formula."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth
from oracle.psumbook_path import psum_gemm


def tiny(K, N, v, m, B, seed, g=-1):
    return synth.generate(synth.custom_case(K, N, v, m, B, seed, g=g))


def frac(a):
    return Fraction(float(a))


def brute_force(inp):
    """Exact rational arithmetic, pure Python loops, straight from the definitions."""
    c = inp.case
    y = [[Fraction(0)] * c.N for _ in range(c.B)]
    T = [[Fraction(0)] * c.N for _ in range(c.B)]
    for n in range(c.N):
        for kk in range(c.K):
            s = frac(inp.scales[n]) if c.g == -1 else frac(inp.scales[n, kk // c.g])
            j, k = divmod(kk, c.v)
            w = Fraction(0)
            for cb in range(c.m):
                w += frac(inp.codebooks[cb, inp.codes[cb, n, j], k])
            w *= s
            for b in range(c.B):
                t = frac(inp.x[b, kk]) * w
                y[b][n] += t
                T[b][n] += abs(t)
    return y, T


# Fig. 2 illustrates a 4 x 32 matrix with v = 8; it is one of the brute-force shapes.
@pytest.mark.parametrize("K,N,v,m,B", [(32, 4, 8, 1, 1), (16, 5, 4, 1, 2), (16, 3, 8, 2, 3),
                                      (24, 7, 4, 3, 1), (8, 1, 8, 4, 2), (12, 6, 4, 2, 1), (32, 3, 16, 3, 2), (48, 2, 16, 4, 1)])
def test_brute_force_exact_rational(K, N, v, m, B):
    inp = tiny(K, N, v, m, B, 1000 + K + N)
    y, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    yb, Tb = brute_force(inp)
    for b in range(B):
        for n in range(N):
            assert abs(y[b, n] - float(yb[b][n])) <= 4e-16 * float(Tb[b][n]) * K
            assert abs(T[b, n] - float(Tb[b][n])) <= 4e-16 * float(Tb[b][n]) * K


@pytest.mark.parametrize("K,N,v,m,B", [(512, 512, 8, 1, 1), (256, 65, 4, 1, 3), (1024, 130, 8, 2, 2),
                                      (328, 33, 8, 3, 1), (136, 17, 4, 4, 2)])
def test_gather_identity_and_op_counts(K, N, v, m, B):
    """Section 3: gathering Psums by code and accumulating equals the dequantized
    product; the work done is the two terms of Eq. 3."""
    inp = tiny(K, N, v, m, B, 77)
    y, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    y2, cnt = psum_gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    assert np.all(np.abs(y - y2) <= 1e-12 * T)
    assert cnt["build_macs"] == m * 256 * v * (K // v) * B     # C_build of Eq. 3
    assert cnt["gathers"] == m * N * (K // v) * B             # C_read of Eq. 3


def test_psumbook_eq2_brute_force():
    inp = tiny(24, 2, 4, 2, 2, 5)
    P = oracle.psumbook(inp.x, inp.codebooks)
    assert P.shape == (2, 2, 6, 256)
    for b in range(2):
        for c in range(2):
            for j in range(6):
                for i in range(0, 256, 7):
                    want = sum(frac(inp.codebooks[c, i, k]) * frac(inp.x[b, 4 * j + k]) for k in range(4))
                    assert abs(P[b, c, j, i] - float(want)) <= 1e-15


def test_psumbook_one_hot_centroids_copy_x_all_half_patterns():
    """With C[i] = e_{i mod v}, Eq. 2 gives P[j][i] = x[v j + i mod v] exactly.
    x runs over every finite binary16 bit pattern, so this also pins the
    half -> double conversion (subnormals included)."""
    v = 8
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = bits.view(np.float16)
    x = x[np.isfinite(x)]
    assert x.size % v == 0
    x = x.reshape(1, -1)
    cb = np.zeros((1, 256, v), np.float16)
    cb[0, np.arange(256), np.arange(256) % v] = 1.0
    P = oracle.psumbook(x, cb)
    xr = x.astype(np.float64).reshape(-1, v)
    want = xr[:, np.arange(256) % v]
    assert np.array_equal(P[0, 0], want)


def test_psumbook_one_hot_x_reads_codebook():
    """x = e_k inside every sub-vector makes P[c][j][i] = C[c][i][k]: pins the
    conversion and indexing of the codebook operand."""
    v, m, J = 4, 2, 3
    rng = np.random.default_rng(3)
    cb = rng.standard_normal((m, 256, v)).astype(np.float16)
    cb[0, :8, 0] = np.array([6e-8, -6e-8, 6.1e-5, 65504, -65504, 0.0, -0.0, 1e-7], np.float16)
    for k in range(v):
        x = np.zeros((1, J * v), np.float16)
        x[0, k::v] = 1.0
        P = oracle.psumbook(x, cb)
        for j in range(J):
            assert np.array_equal(P[0, :, j, :], cb[:, :, k].astype(np.float64))


def test_zero_codebook_gives_zero_and_drops_out():
    inp = tiny(64, 9, 8, 2, 2, 11)
    z = np.zeros_like(inp.codebooks)
    y, T = oracle.gemm(inp.x, inp.codes, z, inp.scales)
    assert np.all(y == 0) and np.all(T == 0)
    cb = inp.codebooks.copy()
    cb[1] = 0
    y2, _ = oracle.gemm(inp.x, inp.codes, cb, inp.scales)
    y1, _ = oracle.gemm(inp.x, inp.codes[:1], inp.codebooks[:1], inp.scales)
    assert np.array_equal(y1, y2)


def test_one_hot_centroids_gather_sum_of_x():
    """C[i] = e_{i mod v}  =>  y[b][n] = s[n] * sum_j x[b][v j + code[n][j] mod v]."""
    v = 8
    inp = tiny(128, 21, v, 1, 2, 13)
    cb = np.zeros((1, 256, v), np.float16)
    cb[0, np.arange(256), np.arange(256) % v] = 1.0
    y, _ = oracle.gemm(inp.x, inp.codes, cb, inp.scales)
    J = 128 // v
    pos = v * np.arange(J)[None, :] + (inp.codes[0].astype(np.int64) % v)        # [N][J]
    for b in range(2):
        want = inp.x[b].astype(np.float64)[pos]                                   # [N][J]
        want = np.array([sum(Fraction(float(t)) for t in row) for row in want], dtype=object)
        want = np.array([float(w * Fraction(float(s))) for w, s in zip(want, inp.scales)])
        assert np.allclose(y[b], want, rtol=1e-14, atol=1e-14)


def sign_codebook(v, lo):
    """Centroid i has element k equal to +1 if bit k of i is set, else lo
    (lo = -1: binary-coded, lo = 0: uniform {0,1}; Section 5, LUT paragraph)."""
    i = np.arange(256)[:, None]
    k = np.arange(v)[None, :]
    return np.where((i >> k) & 1, 1.0, lo).astype(np.float16)[None]


@pytest.mark.parametrize("lo", [-1.0, 0.0])
def test_sign_codebook_equals_integer_matrix_product(lo):
    """With a +-1 (or 0/1) codebook W is an integer matrix; with integer x the
    product is an exact integer computable by an unrelated int64 routine."""
    v, K, N, B = 8, 256, 40, 3
    rng = np.random.default_rng(17)
    codes = rng.integers(0, 256, (1, N, K // v), dtype=np.uint8)
    x = rng.integers(-8, 9, (B, K)).astype(np.float16)
    s = np.ones(N, np.float16)
    # the integer matrix, built from the bits of the codes without any codebook lookup
    bits = ((codes[0][:, :, None] >> np.arange(v)[None, None, :]) & 1).reshape(N, K).astype(np.int64)
    S = bits if lo == 0.0 else 2 * bits - 1
    want = x.astype(np.int64) @ S.T
    y, T = oracle.gemm(x, codes, sign_codebook(v, lo), s)
    assert np.array_equal(y, want.astype(np.float64))
    assert np.array_equal(T, (np.abs(x.astype(np.int64)) @ np.abs(S).T).astype(np.float64))


def test_scale_linearity_power_of_two():
    inp = tiny(64, 12, 4, 2, 2, 19)
    y, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    s2 = inp.scales.copy()
    s2[::2] *= 2
    y2, T2 = oracle.gemm(inp.x, inp.codes, inp.codebooks, s2)
    assert np.array_equal(y2[:, ::2], 2 * y[:, ::2]) and np.array_equal(y2[:, 1::2], y[:, 1::2])
    assert np.array_equal(T2[:, ::2], 2 * T[:, ::2])


def test_row_permutation_equivariance():
    inp = tiny(96, 31, 8, 2, 2, 23)
    perm = np.random.default_rng(1).permutation(31)
    y, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    yp, _ = oracle.gemm(inp.x, inp.codes[:, perm, :], inp.codebooks, inp.scales[perm])
    assert np.array_equal(yp, y[:, perm])


def test_constant_codes_make_rows_proportional_to_scale():
    inp = tiny(64, 10, 4, 1, 1, 29)
    codes = np.full_like(inp.codes, 37)
    y, _ = oracle.gemm(inp.x, codes, inp.codebooks, inp.scales)
    r = y[0] / inp.scales.astype(np.float64)
    assert np.allclose(r, r[0], rtol=1e-14)
    # and that constant is the dot product of x with the tiled centroid 37
    w = np.tile(inp.codebooks[0, 37].astype(np.float64), 64 // 4)
    assert np.isclose(r[0], float(np.dot(inp.x[0].astype(np.float64), w)), rtol=1e-13)


def test_sub_vector_position_matters():
    """Moving one code to another sub-vector j changes y by the difference of two
    specific Psums: catches a transposed or mis-strided code index."""
    inp = tiny(32, 3, 8, 1, 1, 31)
    P = oracle.psumbook(inp.x, inp.codebooks)[0, 0]        # [J][256]
    y0, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    codes = inp.codes.copy()
    n, j, new = 1, 2, (int(inp.codes[0, 1, 2]) + 91) % 256
    old = int(codes[0, n, j])
    codes[0, n, j] = new
    y1, _ = oracle.gemm(inp.x, codes, inp.codebooks, inp.scales)
    delta = float(inp.scales[n]) * (P[j, new] - P[j, old])
    assert np.isclose(y1[0, n] - y0[0, n], delta, rtol=1e-9, atol=1e-15)
    assert np.array_equal(np.delete(y1, n, axis=1), np.delete(y0, n, axis=1))


def test_dequantize_consistent_with_gemm():
    inp = tiny(64, 14, 8, 3, 2, 37)
    W = oracle.dequantize(inp.codes, inp.codebooks, inp.scales)
    y, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    assert np.allclose(inp.x.astype(np.float64) @ W.T, y, rtol=1e-12, atol=1e-14)
    # element (n, v j + k) of W against a hand lookup
    n, j, k = 5, 3, 6
    want = float(inp.scales[n]) * sum(float(inp.codebooks[c, inp.codes[c, n, j], k]) for c in range(3))
    assert np.isclose(W[n, 8 * j + k], want, rtol=1e-15)


def test_rejects_bad_shapes():
    inp = tiny(32, 4, 8, 1, 1, 41)
    with pytest.raises(ValueError):
        oracle.gemm(inp.x[:, :31], inp.codes, inp.codebooks, inp.scales)


# ---- normalisation groups along K (Section 2.2, Step 1: g/v vectors share one scale) ----

@pytest.mark.parametrize("K,N,v,m,B,g", [(32, 4, 8, 1, 1, 8), (32, 3, 8, 2, 2, 16), (24, 5, 4, 1, 1, 12),
                                        (16, 2, 4, 3, 2, 4), (64, 3, 8, 2, 1, 32)])
def test_groups_brute_force_exact_rational(K, N, v, m, B, g):
    inp = tiny(K, N, v, m, B, 2000 + K + g, g=g)
    y, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    yb, Tb = brute_force(inp)
    for b in range(B):
        for n in range(N):
            assert abs(y[b, n] - float(yb[b][n])) <= 4e-16 * float(Tb[b][n]) * K
            assert abs(T[b, n] - float(Tb[b][n])) <= 4e-16 * float(Tb[b][n]) * K


@pytest.mark.parametrize("K,N,v,m,B,g", [(512, 65, 8, 2, 2, 128), (256, 33, 4, 1, 1, 32), (384, 20, 8, 3, 1, 8),
                                        (256, 17, 4, 4, 2, 4)])
def test_groups_gather_identity(K, N, v, m, B, g):
    """Scaling each group's gathered partial sum equals the dequantized product."""
    inp = tiny(K, N, v, m, B, 78, g=g)
    y, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    y2, _ = psum_gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    assert np.all(np.abs(y - y2) <= 1e-12 * T)


def test_one_group_per_row_is_the_row_scale():
    """g = K is the row-wise normalisation the paper writes as g = -1."""
    inp = tiny(64, 9, 8, 2, 2, 31)
    y, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    y2, T2 = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales.reshape(-1, 1))
    assert np.array_equal(y, y2) and np.array_equal(T, T2)


def test_equal_group_scales_reduce_to_row_scale():
    inp = tiny(96, 6, 4, 2, 1, 32, g=8)
    row = inp.scales[:, 0].copy()
    y, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, np.repeat(row[:, None], 96 // 8, axis=1))
    y2, T2 = oracle.gemm(inp.x, inp.codes, inp.codebooks, row)
    assert np.all(np.abs(y - y2) <= 1e-13 * T2)


def test_group_scale_linearity_and_locality():
    """Doubling one group's scale adds exactly that group's contribution, which is the
    product over that K range alone; zeroing it removes the range."""
    K, N, v, g = 128, 7, 8, 32
    inp = tiny(K, N, v, 2, 2, 33, g=g)
    y, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    G = 2                                              # the third of four groups
    lo, hi = G * g, (G + 1) * g
    # that group's contribution, computed as a separate, smaller layer with a row-wise scale... per row
    sub_scales = np.ascontiguousarray(inp.scales[:, G])
    part, Tp = oracle.gemm(np.ascontiguousarray(inp.x[:, lo:hi]), np.ascontiguousarray(inp.codes[:, :, lo // v:hi // v]),
                           inp.codebooks, sub_scales)
    doubled = inp.scales.copy(); doubled[:, G] *= np.float16(2)
    y2, T2 = oracle.gemm(inp.x, inp.codes, inp.codebooks, doubled)
    assert np.all(np.abs((y2 - y) - part) <= 1e-13 * T2)
    zeroed = inp.scales.copy(); zeroed[:, G] = 0
    y0, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, zeroed)
    assert np.all(np.abs((y - y0) - part) <= 1e-13 * T2)


def test_group_boundaries_sit_at_multiples_of_g():
    """A scale change in group G must not touch a weight just outside it: with x one-hot at
    position kk, y is the single weight W[n][kk], which carries the scale of group kk // g."""
    K, N, v, g = 48, 4, 4, 12
    inp = tiny(K, N, v, 1, 1, 34, g=g)
    W = oracle.dequantize(inp.codes, inp.codebooks, inp.scales)
    for kk in (0, 11, 12, 23, 24, 35, 36, 47):
        x = np.zeros((1, K), np.float16); x[0, kk] = 1
        y, _ = oracle.gemm(x, inp.codes, inp.codebooks, inp.scales)
        for n in range(N):
            cent = float(inp.codebooks[0, inp.codes[0, n, kk // v], kk % v])
            want = float(inp.scales[n, kk // g]) * cent
            assert y[0, n] == want == W[n, kk]


def test_rejects_bad_group_shapes():
    inp = tiny(32, 4, 8, 1, 1, 35)
    with pytest.raises(ValueError):
        oracle.gemm(inp.x, inp.codes, inp.codebooks, np.ones((4, 3), np.float16))     # 32 / 3 is not whole
    with pytest.raises(RuntimeError):
        oracle.gemm(inp.x, inp.codes, inp.codebooks, np.ones((4, 8), np.float16))     # g = 4 < v
