"""Exact-rational Toom-Cook matrices and the monic-Legendre base change.

Oracle code (test infrastructure): plain ``fractions.Fraction`` arithmetic,
nested Python lists, no blocking, no numpy in the construction.

What is built, with the passage each follows:

* ``toom_cook(m, r, points)``  ->  A^T (m x n), G (n x r), B^T (n x n),
  n = m + r - 1: the Toom-Cook / Winograd construction with linear polynomials
  only, i.e. interpolation at n points (n-1 finite ones plus infinity) followed
  by the matrix-exchange step (Section 3, "Winograd algorithm").  The paper
  names the construction and cites textbooks without printing G, B, A; the
  scaling convention used here (all the 1/N_j factors in G, none in A^T or
  B^T, no sign normalisation) is this repository's reading.
* ``legendre_PT(n)``  ->  P^T, whose row i holds the ascending coefficients of
  the monic ("normalised": leading coefficient 1) Legendre polynomial of
  degree i (Section 4.1; the 6 x 6 instance is printed there).
* ``base_change(...)``  ->  G_P = P G, B_P = P B, A_P = P A and P^{-1}
  (Section 4.1, the sentence after eq. 4).
* ``int_form(T)``  ->  integer numerators N and per-row least common
  denominators rho with T = diag(1/rho) N (used by the quantised pipeline so
  that every stage numerator is an exact integer).
"""
from fractions import Fraction
from math import gcd

INF = "inf"

# Point sets of the benchmark configurations (finite points; infinity is
# implicit and always last).
POINTS = {
    2: [Fraction(0), Fraction(1), Fraction(-1)],
    4: [Fraction(0), Fraction(1), Fraction(-1), Fraction(2), Fraction(-2)],
    6: [Fraction(0), Fraction(1), Fraction(-1), Fraction(2), Fraction(-2),
        Fraction(1, 2), Fraction(-1, 2)],
}


def _zeros(rows, cols):
    return [[Fraction(0) for _ in range(cols)] for _ in range(rows)]


def matmul(A, B):
    rows, inner, cols = len(A), len(B), len(B[0])
    assert len(A[0]) == inner
    C = _zeros(rows, cols)
    for i in range(rows):
        for j in range(cols):
            s = Fraction(0)
            for k in range(inner):
                s += A[i][k] * B[k][j]
            C[i][j] = s
    return C


def transpose(A):
    return [[A[i][j] for i in range(len(A))] for j in range(len(A[0]))]


def identity(n):
    I = _zeros(n, n)
    for i in range(n):
        I[i][i] = Fraction(1)
    return I


def poly_mul_linear(coeffs, root):
    """Ascending coefficients of coeffs(x) * (x - root)."""
    out = [Fraction(0)] * (len(coeffs) + 1)
    for d, c in enumerate(coeffs):
        out[d + 1] += c
        out[d] -= c * root
    return out


def toom_cook(m, r, points):
    """A^T, G, B^T for F(m, r) from ``points`` (n-1 finite values; infinity last).

    With y = A^T [ (G g) .* (B^T d) ] equal to the correlation
    y_i = sum_k d_{i+k} g_k, i < m, for a length-n input d and length-r filter g.
    """
    n = m + r - 1
    pts = [Fraction(p) for p in points]
    if len(pts) != n - 1:
        raise ValueError("need m+r-2 finite points")
    if len(set(pts)) != len(pts):
        raise ValueError("points must be distinct")

    # A^T: evaluation of the degree-(m-1) output monomials at the points.
    AT = _zeros(m, n)
    for i in range(m):
        for j in range(n - 1):
            AT[i][j] = pts[j] ** i
    AT[m - 1][n - 1] = Fraction(1)

    # G: filter evaluated at the points, scaled by the Lagrange denominators.
    G = _zeros(n, r)
    for j in range(n - 1):
        Nj = Fraction(1)
        for k in range(n - 1):
            if k != j:
                Nj *= pts[j] - pts[k]
        for k in range(r):
            G[j][k] = pts[j] ** k / Nj
    G[n - 1][r - 1] = Fraction(1)

    # B^T: row j = coefficients of prod_{k != j} (x - p_k); the infinity row
    # holds the coefficients of the full product prod_k (x - p_k).
    BT = _zeros(n, n)
    for j in range(n - 1):
        poly = [Fraction(1)]
        for k in range(n - 1):
            if k != j:
                poly = poly_mul_linear(poly, pts[k])
        for d, c in enumerate(poly):
            BT[j][d] = c
    poly = [Fraction(1)]
    for k in range(n - 1):
        poly = poly_mul_linear(poly, pts[k])
    for d, c in enumerate(poly):
        BT[n - 1][d] = c
    return AT, G, BT


def legendre_PT(n):
    """P^T (n x n): row i = ascending coefficients of the monic Legendre p_i.

    p_0 = 1, p_1 = x, p_{k+1} = x p_k - k^2 / (4 k^2 - 1) p_{k-1}.
    """
    rows = []
    for i in range(n):
        if i == 0:
            poly = [Fraction(1)]
        elif i == 1:
            poly = [Fraction(0), Fraction(1)]
        else:
            k = i - 1
            shifted = [Fraction(0)] + rows[i - 1]
            coef = Fraction(k * k, 4 * k * k - 1)
            poly = list(shifted)
            for d, c in enumerate(rows[i - 2]):
                poly[d] -= coef * c
        rows.append(poly)
    PT = _zeros(n, n)
    for i, poly in enumerate(rows):
        for d, c in enumerate(poly):
            PT[i][d] = c
    return PT


def chebyshev_PT(n):
    """Row i = ascending coefficients of the monic Chebyshev polynomial of the
    first kind: t_0 = 1, t_1 = x, t_2 = x^2 - 1/2, t_{k+1} = x t_k - t_{k-1} / 4
    (the classical T_k divided by its leading coefficient 2^{k-1})."""
    rows = []
    for i in range(n):
        if i == 0:
            poly = [Fraction(1)]
        elif i == 1:
            poly = [Fraction(0), Fraction(1)]
        else:
            coef = Fraction(1, 2) if i == 2 else Fraction(1, 4)
            poly = [Fraction(0)] + rows[i - 1]
            for d, c in enumerate(rows[i - 2]):
                poly[d] -= coef * c
        rows.append(poly)
    PT = _zeros(n, n)
    for i, poly in enumerate(rows):
        for d, c in enumerate(poly):
            PT[i][d] = c
    return PT


def hermite_PT(n):
    """Row i = ascending coefficients of the monic (probabilists') Hermite
    polynomial: he_0 = 1, he_1 = x, he_{k+1} = x he_k - k he_{k-1}."""
    rows = []
    for i in range(n):
        if i == 0:
            poly = [Fraction(1)]
        elif i == 1:
            poly = [Fraction(0), Fraction(1)]
        else:
            k = i - 1
            poly = [Fraction(0)] + rows[i - 1]
            for d, c in enumerate(rows[i - 2]):
                poly[d] -= k * c
        rows.append(poly)
    PT = _zeros(n, n)
    for i, poly in enumerate(rows):
        for d, c in enumerate(poly):
            PT[i][d] = c
    return PT


def base_PT(n, base):
    return {"canonical": identity, "legendre": legendre_PT, "chebyshev": chebyshev_PT,
            "hermite": hermite_PT}[base](n)


def inverse(A):
    """Gauss-Jordan inverse in exact rationals."""
    n = len(A)
    M = [list(row) + idrow for row, idrow in zip(A, identity(n))]
    for col in range(n):
        piv = None
        for rr in range(col, n):
            if M[rr][col] != 0:
                piv = rr
                break
        if piv is None:
            raise ValueError("singular matrix")
        M[col], M[piv] = M[piv], M[col]
        pv = M[col][col]
        M[col] = [v / pv for v in M[col]]
        for rr in range(n):
            if rr != col and M[rr][col] != 0:
                f = M[rr][col]
                M[rr] = [a - f * b for a, b in zip(M[rr], M[col])]
    return [row[n:] for row in M]


class Matrices:
    """All stage matrices of one F(m, r) instance, as lists of Fractions."""

    def __init__(self, m, r, points=None, base="legendre"):
        self.m, self.r, self.n = m, r, m + r - 1
        pts = POINTS[m] if points is None else points
        self.points = [Fraction(p) for p in pts]
        self.AT, self.G, self.BT = toom_cook(m, r, self.points)
        n = self.n
        self.PT = base_PT(n, base)
        self.PinvT = inverse(self.PT)
        self.P = transpose(self.PT)
        self.Pinv = transpose(self.PinvT)
        A = transpose(self.AT)          # n x m
        B = transpose(self.BT)          # n x n
        # Section 4.1: G_P = P G, B_P = P B, A_P = P A.
        self.GP = matmul(self.P, self.G)            # n x r
        self.BPT = transpose(matmul(self.P, B))     # n x n  (= B^T P^T)
        self.APT = transpose(matmul(self.P, A))     # m x n  (= A^T P^T)


def row_lcd(row):
    l = 1
    for v in row:
        d = Fraction(v).denominator
        l = l * d // gcd(l, d)
    return l


def int_form(T):
    """T = diag(1/rho) N with rho_i the least common denominator of row i."""
    N, rho = [], []
    for row in T:
        l = row_lcd(row)
        rho.append(l)
        N.append([int(v * l) for v in row])
    return N, rho


def lcd(T):
    l = 1
    for row in T:
        rl = row_lcd(row)
        l = l * rl // gcd(l, rl)
    return l


def nnz(T):
    return sum(1 for row in T for v in row if v != 0)


def max_abs_row_sum_int(T):
    """max_i sum_j |N_ij| of the per-row integer form."""
    N, _ = int_form(T)
    return max(sum(abs(v) for v in row) for row in N)
