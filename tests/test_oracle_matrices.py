"""Pins for oracle/matrices.py: printed values, library cross-checks, identities."""
import os
import random
from fractions import Fraction

import numpy as np
import pytest

from oracle import matrices as mx
from oracle import winograd as wg

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_matrix(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([Fraction(tok) for tok in line.split()])
    return rows


def read_counts():
    out = {}
    with open(os.path.join(GOLDEN, "counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                out[k] = v
    return out


def read_blocks(name):
    blocks, cur = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            if line.startswith("["):
                cur = blocks.setdefault(line.strip("[]"), [])
            else:
                cur.append([Fraction(tok) for tok in line.split()])
    return blocks


def test_F43_equals_the_published_matrix_set():
    """The construction (all Lagrange denominators in G, no sign normalisation) reproduces
    the widely used F(4x4,3x3) matrices entry for entry."""
    pub = read_blocks("toomcook_F43_published.txt")
    M = mx.Matrices(4, 3)
    assert M.BT == pub["BT"] and M.G == pub["G"] and M.AT == pub["AT"]


def test_F23_equals_the_published_set_up_to_row_signs():
    """For F(2x2,3x3) the published matrices (B^T rows [1,0,-1,0], [0,1,1,0], [0,-1,1,0],
    [0,1,0,-1]; G rows [1,0,0], [1/2,1/2,1/2], [1/2,-1/2,1/2], [0,0,1]; A^T rows [1,1,1,0],
    [0,1,-1,-1]) differ from this construction only by a sign on the rows of points 0 and
    infinity, applied to G (or A^T) and B^T together, which leaves every product unchanged."""
    F = Fraction
    pub_BT = [[1, 0, -1, 0], [0, 1, 1, 0], [0, -1, 1, 0], [0, 1, 0, -1]]
    pub_G = [[F(1), 0, 0], [F(1, 2), F(1, 2), F(1, 2)], [F(1, 2), F(-1, 2), F(1, 2)], [0, 0, F(1)]]
    pub_AT = [[1, 1, 1, 0], [0, 1, -1, -1]]
    M = mx.Matrices(2, 3)
    for j in range(4):
        sb = 1 if M.BT[j] == [F(v) for v in pub_BT[j]] else -1
        assert M.BT[j] == [sb * F(v) for v in pub_BT[j]]
        sg = 1 if M.G[j] == [F(v) for v in pub_G[j]] else -1
        assert M.G[j] == [sg * F(v) for v in pub_G[j]]
        sa = 1 if [M.AT[i][j] for i in range(2)] == [F(pub_AT[i][j]) for i in range(2)] else -1
        assert [M.AT[i][j] for i in range(2)] == [sa * F(pub_AT[i][j]) for i in range(2)]
        assert sb * sg * sa == 1                   # the three signs of a point cancel


def test_PT_equals_printed_matrix():
    # Section 4.1, first displayed matrix.
    assert mx.legendre_PT(6) == read_matrix("legendre_PT_6x6.txt")


def test_PinvT_equals_printed_matrix():
    # Section 4.1, second displayed matrix.
    assert mx.inverse(mx.legendre_PT(6)) == read_matrix("legendre_PinvT_6x6.txt")
    M = mx.Matrices(4, 3)
    assert M.PinvT == read_matrix("legendre_PinvT_6x6.txt")
    assert mx.matmul(M.PT, M.PinvT) == mx.identity(6)


def test_PT_4x4_is_leading_block():
    full = read_matrix("legendre_PT_6x6.txt")
    assert mx.legendre_PT(4) == [row[:4] for row in full[:4]]


def test_nnz_counts_of_P():
    c = read_counts()
    assert mx.nnz(mx.legendre_PT(4)) == int(c["nnz_P_4x4"])
    assert mx.nnz(mx.legendre_PT(6)) == int(c["nnz_P_6x6"])


@pytest.mark.parametrize("n", [4, 6, 8])
def test_PT_rows_are_monic_legendre_polynomials(n):
    """Independent library check, including the rows the paper does not print."""
    from numpy.polynomial import legendre
    PT = mx.legendre_PT(n)
    for i in range(n):
        coef = legendre.leg2poly([0] * i + [1])          # ascending powers
        coef = coef / coef[-1]                             # make it monic
        got = np.array([float(v) for v in PT[i][:i + 1]])
        assert np.allclose(got, coef, rtol=1e-12, atol=1e-12)
        assert PT[i][i] == 1
        assert all(v == 0 for v in PT[i][i + 1:])


@pytest.mark.parametrize("n", [4, 6, 8])
def test_legendre_rows_are_orthogonal_on_minus1_1(n):
    """int_{-1}^{1} p_i p_j dx = 0 for i != j, exactly (monomial integrals)."""
    PT = mx.legendre_PT(n)
    for i in range(n):
        for j in range(i):
            s = Fraction(0)
            for a, ca in enumerate(PT[i]):
                for b, cb in enumerate(PT[j]):
                    if (a + b) % 2 == 0:
                        s += ca * cb * Fraction(2, a + b + 1)
            assert s == 0


def test_multiplication_counts():
    c = read_counts()
    # (o+k-1)^2 multiplications for o^2 outputs (Section 1).
    assert Fraction((4 + 3 - 1) ** 2, 16) == Fraction(c["mults_per_output_F4_toomcook"])
    assert round(49 / 16, 2) == float(c["mults_per_output_F4_superlinear"])
    for m, expect in ((2, Fraction(4)), (4, Fraction(9, 4)), (6, Fraction(16, 9))):
        M = mx.Matrices(m, 3)
        assert Fraction(len(M.BT) * len(M.BT[0]), m * m) == expect


def _corr1d(d, g, m):
    return [sum(d[i + k] * g[k] for k in range(len(g))) for i in range(m)]


@pytest.mark.parametrize("m", [2, 4, 6])
def test_toom_cook_1d_is_correlation_exactly(m):
    rnd = random.Random(m)
    M = mx.Matrices(m, 3)
    n = M.n
    for _ in range(5):
        d = [Fraction(rnd.randint(-127, 127)) for _ in range(n)]
        g = [Fraction(rnd.randint(-127, 127)) for _ in range(3)]
        Gg = [sum(M.G[j][k] * g[k] for k in range(3)) for j in range(n)]
        Bd = [sum(M.BT[j][k] * d[k] for k in range(n)) for j in range(n)]
        y = [sum(M.AT[i][j] * Gg[j] * Bd[j] for j in range(n)) for i in range(m)]
        assert y == _corr1d(d, g, m)


@pytest.mark.parametrize("m,r,pts", [(3, 2, [0, 1, -1]), (2, 5, [0, 1, -1, 2, -2]),
                                     (4, 3, [0, 1, -1, Fraction(1, 2), -2])])
def test_toom_cook_other_sizes_and_points(m, r, pts):
    rnd = random.Random(7)
    AT, G, BT = mx.toom_cook(m, r, pts)
    n = m + r - 1
    d = [Fraction(rnd.randint(-9, 9)) for _ in range(n)]
    g = [Fraction(rnd.randint(-9, 9)) for _ in range(r)]
    Gg = [sum(G[j][k] * g[k] for k in range(r)) for j in range(n)]
    Bd = [sum(BT[j][k] * d[k] for k in range(n)) for j in range(n)]
    y = [sum(AT[i][j] * Gg[j] * Bd[j] for j in range(n)) for i in range(m)]
    assert y == _corr1d(d, g, m)


def test_toom_cook_rejects_bad_points():
    with pytest.raises(ValueError):
        mx.toom_cook(2, 3, [0, 1, 1])
    with pytest.raises(ValueError):
        mx.toom_cook(2, 3, [0, 1])


@pytest.mark.parametrize("m", [2, 4, 6])
def test_2d_tile_eq3_and_eq4_equal_direct_exactly(m):
    rnd = random.Random(10 + m)
    M = mx.Matrices(m, 3)
    n = M.n
    X = [[Fraction(rnd.randint(-127, 127)) for _ in range(n)] for _ in range(n)]
    Wk = [[Fraction(rnd.randint(-127, 127)) for _ in range(3)] for _ in range(3)]
    want = wg.tile_direct_fraction(X, Wk, m, 3)
    assert wg.tile_eq3_fraction(X, Wk, M) == want
    assert wg.tile_eq4_fraction(X, Wk, M) == want


@pytest.mark.parametrize("m", [2, 4, 6])
def test_legendre_factorisation_identities(m):
    """P^{-1} G_P = G, B_P^T P^{-T} = B^T, A_P^T P^{-T} = A^T (Section 4.1)."""
    M = mx.Matrices(m, 3)
    assert mx.matmul(M.Pinv, M.GP) == M.G
    assert mx.matmul(M.BPT, M.PinvT) == M.BT
    assert mx.matmul(M.APT, M.PinvT) == M.AT
    # eq. 2 == eq. 1 on an integer filter
    rnd = random.Random(3)
    Wk = [[Fraction(rnd.randint(-127, 127)) for _ in range(3)] for _ in range(3)]
    eq1 = mx.matmul(mx.matmul(M.G, Wk), mx.transpose(M.G))
    inner = mx.matmul(mx.matmul(M.GP, Wk), mx.transpose(M.GP))
    eq2 = mx.matmul(mx.matmul(M.Pinv, inner), M.PinvT)
    assert eq1 == eq2


def test_eq4_as_printed_is_not_a_convolution():
    """With P (not P^{-1}) as the right factor of the inner input bracket,
    eq. 4 differs from eq. 3: the reading with P^{-1} is the consistent one."""
    M = mx.Matrices(4, 3)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((1, 4, 4, 2))
    w = rng.standard_normal((2, 2, 3, 3))
    y3 = wg.conv_eq3(x, w, M)
    assert np.allclose(wg.conv_eq4(x, w, M), y3, rtol=1e-9, atol=1e-9)
    assert not np.allclose(wg.conv_eq4(x, w, M, literal_print=True), y3, rtol=1e-2, atol=1e-2)


def test_int_form_roundtrip_and_row_lcds():
    M = mx.Matrices(4, 3)
    for T in (M.G, M.BT, M.AT, M.PT, M.PinvT, M.GP, M.BPT, M.APT):
        N, rho = mx.int_form(T)
        for i, row in enumerate(T):
            for j, v in enumerate(row):
                assert Fraction(N[i][j], rho[i]) == v
            g = 0
            from math import gcd
            for v in N[i] + [rho[i]]:
                g = gcd(g, abs(v))
            assert g == 1                      # rho_i is the *least* common denominator


@pytest.mark.parametrize("n", [4, 6, 8])
def test_chebyshev_and_hermite_rows_against_numpy(n):
    """The other bases Section 4.1 names, pinned to library conversions."""
    from numpy.polynomial import chebyshev, hermite_e
    for rows, conv in ((mx.chebyshev_PT(n), chebyshev.cheb2poly),
                       (mx.hermite_PT(n), hermite_e.herme2poly)):
        for i in range(n):
            coef = conv([0] * i + [1])
            coef = coef / coef[-1]
            got = np.array([float(v) for v in rows[i][:i + 1]])
            assert np.allclose(got, coef, rtol=1e-12, atol=1e-12)
            assert rows[i][i] == 1 and all(v == 0 for v in rows[i][i + 1:])


@pytest.mark.parametrize("base", ["chebyshev", "hermite"])
def test_other_bases_leave_the_convolution_unchanged(base):
    M = mx.Matrices(4, 3, base=base)
    assert mx.matmul(M.Pinv, M.GP) == M.G
    assert mx.matmul(M.BPT, M.PinvT) == M.BT
    assert mx.matmul(M.APT, M.PinvT) == M.AT
    rnd = random.Random(5)
    X = [[Fraction(rnd.randint(-127, 127)) for _ in range(6)] for _ in range(6)]
    Wk = [[Fraction(rnd.randint(-127, 127)) for _ in range(3)] for _ in range(3)]
    assert wg.tile_eq4_fraction(X, Wk, M) == wg.tile_direct_fraction(X, Wk, 4, 3)
