// Exact rational arithmetic and the Toom-Cook / Legendre matrix construction,
// written as constexpr C++ so that the very same code serves
//   * the host entry point wino_make_matrices (run time, any points), and
//   * the HIP kernels, which instantiate the standard point sets at compile
//     time and read the integer forms as constant expressions.
//
// Construction (Section 3, "Winograd algorithm": Toom-Cook = interpolation at
// n points followed by the matrix-exchange step; Section 4.1 for the Legendre
// base change).  With finite points p_0..p_{n-2} and the point at infinity
// last, n = m + r - 1:
//   A^T (m x n):  A^T[i][j] = p_j^i,            infinity column = e_{m-1}
//   G   (n x r):  G[j][k]   = p_j^k / N_j,      N_j = prod_{k!=j} (p_j - p_k),
//                 infinity row = e_{r-1}
//   B^T (n x n):  row j = ascending coefficients of prod_{k!=j} (x - p_k),
//                 infinity row = coefficients of prod_k (x - p_k)
//   P^T (n x n):  row i = ascending coefficients of the monic Legendre
//                 polynomial p_i, p_{k+1} = x p_k - k^2/(4k^2-1) p_{k-1}
//   G_P = P G,  B_P = P B,  A_P = P A  (so B_P^T = B^T P^T, A_P^T = A^T P^T).
// Every rational is kept reduced with a positive denominator; any int64
// overflow clears the `ok` flag of the result instead of wrapping.
#pragma once
#include <cstdint>

namespace wino {

constexpr int kMaxN = 8;   // largest supported Winograd tile edge m + r - 1

constexpr int64_t cabs64(int64_t v) { return v < 0 ? -v : v; }

constexpr int64_t cgcd(int64_t a, int64_t b) {
  a = cabs64(a);
  b = cabs64(b);
  while (b != 0) {
    int64_t t = a % b;
    a = b;
    b = t;
  }
  return a;
}

struct Rat {
  int64_t num = 0;
  int64_t den = 1;
  bool ok = true;
};

constexpr Rat make_rat(int64_t num, int64_t den, bool ok = true) {
  Rat r;
  if (!ok || den == 0 || num == INT64_MIN || den == INT64_MIN) {
    r.ok = false;
    return r;
  }
  if (den < 0) {
    num = -num;
    den = -den;
  }
  int64_t g = cgcd(num, den);
  if (g > 1) {
    num /= g;
    den /= g;
  }
  r.num = num;
  r.den = den;
  return r;
}

constexpr Rat rat_mul(const Rat& a, const Rat& b) {
  // cross-reduce first so that intermediate products stay small
  int64_t g1 = cgcd(a.num, b.den), g2 = cgcd(b.num, a.den);
  int64_t an = g1 ? a.num / g1 : a.num, bd = g1 ? b.den / g1 : b.den;
  int64_t bn = g2 ? b.num / g2 : b.num, ad = g2 ? a.den / g2 : a.den;
  int64_t n = 0, d = 0;
  bool ovf = __builtin_mul_overflow(an, bn, &n);
  ovf |= __builtin_mul_overflow(ad, bd, &d);
  return make_rat(n, d, a.ok && b.ok && !ovf);
}

constexpr Rat rat_add(const Rat& a, const Rat& b) {
  int64_t g = cgcd(a.den, b.den);
  int64_t bd = b.den / g, ad = a.den / g;
  int64_t t1 = 0, t2 = 0, n = 0, d = 0;
  bool ovf = __builtin_mul_overflow(a.num, bd, &t1);
  ovf |= __builtin_mul_overflow(b.num, ad, &t2);
  ovf |= __builtin_add_overflow(t1, t2, &n);
  ovf |= __builtin_mul_overflow(a.den, bd, &d);
  return make_rat(n, d, a.ok && b.ok && !ovf);
}

constexpr Rat rat_neg(const Rat& a) { return make_rat(-a.num, a.den, a.ok); }
constexpr Rat rat_sub(const Rat& a, const Rat& b) { return rat_add(a, rat_neg(b)); }
constexpr Rat rat_div(const Rat& a, const Rat& b) {
  return rat_mul(a, make_rat(b.den, b.num, b.ok && b.num != 0));
}
constexpr bool rat_eq(const Rat& a, const Rat& b) { return a.num == b.num && a.den == b.den; }
constexpr bool rat_is_zero(const Rat& a) { return a.num == 0; }

struct RMat {
  int rows = 0, cols = 0;
  Rat a[kMaxN][kMaxN] = {};
  bool ok = true;
};

constexpr RMat rmat(int rows, int cols) {
  RMat m;
  m.rows = rows;
  m.cols = cols;
  return m;
}

constexpr bool rmat_ok(const RMat& m) {
  if (!m.ok) return false;
  for (int i = 0; i < m.rows; ++i)
    for (int j = 0; j < m.cols; ++j)
      if (!m.a[i][j].ok) return false;
  return true;
}

constexpr RMat rmat_mul(const RMat& x, const RMat& y) {
  RMat z = rmat(x.rows, y.cols);
  z.ok = x.ok && y.ok && x.cols == y.rows;
  for (int i = 0; i < x.rows; ++i)
    for (int j = 0; j < y.cols; ++j) {
      Rat s;
      for (int k = 0; k < x.cols; ++k)
        if (!rat_is_zero(x.a[i][k]) && !rat_is_zero(y.a[k][j]))
          s = rat_add(s, rat_mul(x.a[i][k], y.a[k][j]));
      z.a[i][j] = s;
    }
  z.ok = z.ok && rmat_ok(z);
  return z;
}

constexpr RMat rmat_transpose(const RMat& x) {
  RMat z = rmat(x.cols, x.rows);
  z.ok = x.ok;
  for (int i = 0; i < x.rows; ++i)
    for (int j = 0; j < x.cols; ++j) z.a[j][i] = x.a[i][j];
  return z;
}

constexpr RMat rmat_identity(int n) {
  RMat z = rmat(n, n);
  for (int i = 0; i < n; ++i) z.a[i][i] = make_rat(1, 1);
  return z;
}

// Gauss-Jordan inverse; a singular input clears ok.
constexpr RMat rmat_inverse(const RMat& x) {
  const int n = x.rows;
  RMat a = x, inv = rmat_identity(n);
  inv.ok = x.ok && x.rows == x.cols;
  for (int col = 0; col < n && inv.ok; ++col) {
    int piv = -1;
    for (int r = col; r < n; ++r)
      if (!rat_is_zero(a.a[r][col])) {
        piv = r;
        break;
      }
    if (piv < 0) {
      inv.ok = false;
      break;
    }
    for (int j = 0; j < n; ++j) {
      Rat t = a.a[col][j];
      a.a[col][j] = a.a[piv][j];
      a.a[piv][j] = t;
      t = inv.a[col][j];
      inv.a[col][j] = inv.a[piv][j];
      inv.a[piv][j] = t;
    }
    Rat pv = a.a[col][col];
    for (int j = 0; j < n; ++j) {
      a.a[col][j] = rat_div(a.a[col][j], pv);
      inv.a[col][j] = rat_div(inv.a[col][j], pv);
    }
    for (int r = 0; r < n; ++r) {
      if (r == col || rat_is_zero(a.a[r][col])) continue;
      Rat f = a.a[r][col];
      for (int j = 0; j < n; ++j) {
        a.a[r][j] = rat_sub(a.a[r][j], rat_mul(f, a.a[col][j]));
        inv.a[r][j] = rat_sub(inv.a[r][j], rat_mul(f, inv.a[col][j]));
      }
    }
  }
  inv.ok = inv.ok && rmat_ok(inv);
  return inv;
}

// poly (ascending, `len` coefficients) times (x - root); result has len + 1.
constexpr void poly_times_linear(Rat* poly, int len, const Rat& root) {
  poly[len] = Rat{};
  for (int d = len; d >= 1; --d) poly[d] = rat_sub(poly[d - 1], rat_mul(poly[d], root));
  poly[0] = rat_neg(rat_mul(poly[0], root));
}

constexpr Rat rat_pow(const Rat& b, int e) {
  Rat r = make_rat(1, 1);
  for (int i = 0; i < e; ++i) r = rat_mul(r, b);
  return r;
}

struct MatrixSet {
  int m = 0, r = 0, n = 0;
  RMat AT, G, BT;          // canonical Toom-Cook matrices
  RMat PT, PinvT, P, Pinv; // monic-Legendre base change and its inverse
  RMat GP, BPT, APT;       // G_P = P G, B_P^T = B^T P^T, A_P^T = A^T P^T
  bool ok = true;
};

constexpr RMat legendre_PT(int n) {
  RMat pt = rmat(n, n);
  for (int i = 0; i < n; ++i) {
    if (i == 0) {
      pt.a[0][0] = make_rat(1, 1);
    } else if (i == 1) {
      pt.a[1][1] = make_rat(1, 1);
    } else {
      const int64_t k = i - 1;
      const Rat coef = make_rat(k * k, 4 * k * k - 1);
      for (int d = 1; d <= i; ++d) pt.a[i][d] = pt.a[i - 1][d - 1];
      for (int d = 0; d <= i - 2; ++d)
        pt.a[i][d] = rat_sub(pt.a[i][d], rat_mul(coef, pt.a[i - 2][d]));
    }
  }
  pt.ok = rmat_ok(pt);
  return pt;
}

// Other classical orthogonal families, also monic (Section 4.1 names them as
// the usual alternatives to Legendre).
//   Chebyshev (first kind): t_0 = 1, t_1 = x, t_2 = x^2 - 1/2, t_{k+1} = x t_k - t_{k-1}/4
//   Hermite (probabilists'): he_0 = 1, he_1 = x, he_{k+1} = x he_k - k he_{k-1}
constexpr RMat recurrence_PT(int n, int family) {
  RMat pt = rmat(n, n);
  for (int i = 0; i < n; ++i) {
    if (i == 0) {
      pt.a[0][0] = make_rat(1, 1);
    } else if (i == 1) {
      pt.a[1][1] = make_rat(1, 1);
    } else {
      const int64_t k = i - 1;
      const Rat coef = family == 2 ? (i == 2 ? make_rat(1, 2) : make_rat(1, 4)) : make_rat(k, 1);
      for (int d = 1; d <= i; ++d) pt.a[i][d] = pt.a[i - 1][d - 1];
      for (int d = 0; d <= i - 2; ++d)
        pt.a[i][d] = rat_sub(pt.a[i][d], rat_mul(coef, pt.a[i - 2][d]));
    }
  }
  pt.ok = rmat_ok(pt);
  return pt;
}

// base: 0 canonical (P = I), 1 monic Legendre, 2 monic Chebyshev, 3 monic Hermite.
constexpr RMat base_PT(int n, int base) {
  if (base == 0) return rmat_identity(n);
  if (base == 1) return legendre_PT(n);
  return recurrence_PT(n, base);
}

// points: n-1 finite rationals (infinity implicit and last).  `base` selects
// the base-change matrix P (see base_PT; 0 makes it the identity: G_P = G, ...).
constexpr MatrixSet make_matrix_set(int m, int r, const Rat* points, int n_finite,
                                    int base = 1) {
  MatrixSet s;
  s.m = m;
  s.r = r;
  s.n = m + r - 1;
  const int n = s.n;
  if (m < 1 || r < 1 || n > kMaxN || n_finite != n - 1) {
    s.ok = false;
    return s;
  }
  for (int i = 0; i < n_finite; ++i) {
    if (!points[i].ok || points[i].den == 0) {
      s.ok = false;
      return s;
    }
    for (int j = 0; j < i; ++j)
      if (rat_eq(make_rat(points[i].num, points[i].den), make_rat(points[j].num, points[j].den))) {
        s.ok = false;
        return s;
      }
  }
  Rat p[kMaxN] = {};
  for (int i = 0; i < n_finite; ++i) p[i] = make_rat(points[i].num, points[i].den);

  s.AT = rmat(m, n);
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n - 1; ++j) s.AT.a[i][j] = rat_pow(p[j], i);
  s.AT.a[m - 1][n - 1] = make_rat(1, 1);

  s.G = rmat(n, r);
  for (int j = 0; j < n - 1; ++j) {
    Rat Nj = make_rat(1, 1);
    for (int k = 0; k < n - 1; ++k)
      if (k != j) Nj = rat_mul(Nj, rat_sub(p[j], p[k]));
    for (int k = 0; k < r; ++k) s.G.a[j][k] = rat_div(rat_pow(p[j], k), Nj);
  }
  s.G.a[n - 1][r - 1] = make_rat(1, 1);

  s.BT = rmat(n, n);
  for (int j = 0; j < n; ++j) {
    Rat poly[kMaxN + 1] = {};
    poly[0] = make_rat(1, 1);
    int len = 1;
    for (int k = 0; k < n - 1; ++k)
      if (k != j) {
        poly_times_linear(poly, len, p[k]);
        ++len;
      }
    for (int d = 0; d < len && d < n; ++d) s.BT.a[j][d] = poly[d];
  }

  s.PT = base_PT(n, base);
  s.PinvT = rmat_inverse(s.PT);
  s.P = rmat_transpose(s.PT);
  s.Pinv = rmat_transpose(s.PinvT);
  s.GP = rmat_mul(s.P, s.G);
  s.BPT = rmat_mul(s.BT, s.PT);
  s.APT = rmat_mul(s.AT, s.PT);
  s.ok = rmat_ok(s.AT) && rmat_ok(s.G) && rmat_ok(s.BT) && rmat_ok(s.PT) && rmat_ok(s.PinvT) &&
         rmat_ok(s.GP) && rmat_ok(s.BPT) && rmat_ok(s.APT);
  return s;
}

// The point sets of the supported F(m x m, 3 x 3) instances.
constexpr MatrixSet standard_matrix_set(int m, int base = 1) {
  if (m == 2) {
    const Rat pts[3] = {make_rat(0, 1), make_rat(1, 1), make_rat(-1, 1)};
    return make_matrix_set(2, 3, pts, 3, base);
  }
  if (m == 4) {
    const Rat pts[5] = {make_rat(0, 1), make_rat(1, 1), make_rat(-1, 1), make_rat(2, 1),
                        make_rat(-2, 1)};
    return make_matrix_set(4, 3, pts, 5, base);
  }
  if (m == 6) {
    const Rat pts[7] = {make_rat(0, 1), make_rat(1, 1),  make_rat(-1, 1), make_rat(2, 1),
                        make_rat(-2, 1), make_rat(1, 2), make_rat(-1, 2)};
    return make_matrix_set(6, 3, pts, 7, base);
  }
  MatrixSet bad;
  bad.ok = false;
  return bad;
}

// Integer form of a stage matrix: T = diag(1/rho) N, rho_i = least common
// denominator of row i.  `rowsum` = max_i sum_j |N_ij| bounds every numerator.
struct IMat {
  int rows = 0, cols = 0;
  int64_t N[kMaxN][kMaxN] = {};
  int64_t rho[kMaxN] = {};
  int64_t rowsum = 0;
  bool ok = true;
};

constexpr IMat int_form(const RMat& t) {
  IMat im;
  im.rows = t.rows;
  im.cols = t.cols;
  im.ok = rmat_ok(t);
  for (int i = 0; i < t.rows && im.ok; ++i) {
    int64_t l = 1;
    for (int j = 0; j < t.cols; ++j) {
      int64_t d = t.a[i][j].den;
      int64_t g = cgcd(l, d);
      if (__builtin_mul_overflow(l / g, d, &l)) im.ok = false;
    }
    im.rho[i] = l;
    int64_t sum = 0;
    for (int j = 0; j < t.cols && im.ok; ++j) {
      int64_t v = 0;
      if (__builtin_mul_overflow(t.a[i][j].num, l / t.a[i][j].den, &v)) im.ok = false;
      im.N[i][j] = v;
      if (__builtin_add_overflow(sum, cabs64(v), &sum)) im.ok = false;
    }
    if (sum > im.rowsum) im.rowsum = sum;
  }
  return im;
}

}  // namespace wino
