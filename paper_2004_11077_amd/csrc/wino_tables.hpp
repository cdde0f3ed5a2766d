// Compile-time integer forms of the stage matrices of the standard
// F(m x m, 3 x 3) instances, built by the same constexpr code that serves
// wino_make_matrices.  Kernels read the entries as constant expressions, so
// zeros vanish and small coefficients become shifts and adds.
#pragma once
#include <type_traits>

#include "wino_rational.hpp"

namespace wino {

constexpr bool rmat_equal(const RMat& a, const RMat& b) {
  if (a.rows != b.rows || a.cols != b.cols) return false;
  for (int i = 0; i < a.rows; ++i)
    for (int j = 0; j < a.cols; ++j)
      if (!rat_eq(a.a[i][j], b.a[i][j])) return false;
  return true;
}

// BASE: the polynomial base of the two-bracket forms (Section 4.1): 1 monic Legendre (the
// paper's), 2 monic Chebyshev, 3 monic Hermite (the alternatives it names).  G, B^T, A^T do
// not depend on it.
template <int M, int BASE = 1>
struct Tab {
  static constexpr MatrixSet ms = standard_matrix_set(M, BASE);
  static_assert(ms.ok, "standard matrix set overflowed");
  // Section 4.1 identities: each Legendre bracket pair multiplies out to the
  // canonical matrix, so eq. 4 without inner casts is eq. 3.
  static_assert(rmat_equal(rmat_mul(ms.BPT, ms.PinvT), ms.BT));
  static_assert(rmat_equal(rmat_mul(ms.APT, ms.PinvT), ms.AT));
  static_assert(rmat_equal(rmat_mul(ms.Pinv, ms.GP), ms.G));

  static constexpr IMat G = int_form(ms.G);
  static constexpr IMat BT = int_form(ms.BT);
  static constexpr IMat AT = int_form(ms.AT);
  static constexpr IMat PinvT = int_form(ms.PinvT);
  static constexpr IMat Pinv = int_form(ms.Pinv);
  static constexpr IMat GP = int_form(ms.GP);
  static constexpr IMat BPT = int_form(ms.BPT);
  static constexpr IMat APT = int_form(ms.APT);
  static_assert(G.ok && BT.ok && AT.ok && PinvT.ok && Pinv.ok && GP.ok && BPT.ok && APT.ok);
};

// Numerators of a stage with |input| <= in_max are bounded by
// in_max * rowsum^2; pick the narrowest exact accumulator.
constexpr bool fits_bits(const IMat& t, int64_t in_max, int bits) {
  __int128 b = (__int128)in_max * t.rowsum * t.rowsum;
  return b < ((__int128)1 << (bits - 1));
}

// Storage of a stage's results: int32_t where every entry fits, else 8-byte
// slots (the transforms pick the arithmetic of each entry by its own bound).
template <const IMat& T, int64_t IN_MAX>
using acc_t = std::conditional_t<fits_bits(T, IN_MAX, 32), int32_t, int64_t>;

// Sum of the absolute values of row i: |(N x)[i]| <= in_max * row_abs(i).
constexpr int64_t row_abs(const IMat& t, int i) {
  int64_t s = 0;
  for (int a = 0; a < t.cols; ++a) s += t.N[i][a] < 0 ? -t.N[i][a] : t.N[i][a];
  return s;
}

// Largest |M| the contraction may produce when it is passed on unquantised
// (bits_hadamard = 32): C * 127^2 must stay below 2^24 so that its fp32
// conversion is exact.
constexpr int64_t kMaxAccUnquantised = (int64_t)1 << 24;
constexpr int kMaxChannelsExact = 1040;   // 1040 * 127 * 127 < 2^24

}  // namespace wino
