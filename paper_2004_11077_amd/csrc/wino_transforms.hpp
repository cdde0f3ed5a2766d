// Transform kernels (gfx950) of the quantised Winograd convolution layer,
// templated on the output tile edge M; one translation unit per M instantiates
// PerM<M>.  Stages of eq. 3 / eq. 4 covered here:
//   weight transform   eq. 1 / eq. 2
//   input transform    input bracket of eq. 3 / eq. 4
//   output transform   output bracket of eq. 3 / eq. 4
// Every cast is  q = clamp(rint(float(num) * mult), +-qmax)  on exact integer
// numerators num = N x N^T (N = integer form of the stage matrix).
#pragma once
#include "wino_kernels.hpp"
#include "wino_tables.hpp"

namespace wino {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

template <int I>
using IC = std::integral_constant<int, I>;

template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(IC<B>{});
    static_for<B + 1, E>(f);
  }
}

// The 24-bit signed multiply (full rate, v_mul_i32_i24 / v_mad_i32_i24): the
// low 32 bits of the product of the operands' low 24 bits.
extern "C" __device__ int llvm_mul_i24(int, int) __asm("llvm.amdgcn.mul.i24.i32");

// A compile-time constant parked in a scalar register.  VOP3 instructions on
// gfx9-class ISAs take no 32-bit literal, so a multiply-add by a large literal
// is otherwise split into a literal multiply and a separate add; with the
// constant in an SGPR it stays one v_mad_i32_i24.
template <int32_t CF>
__device__ __forceinline__ int32_t sconst() {
  if constexpr (CF >= -16 && CF <= 64) {
    return CF;                                   // inline constant, free
  } else {
    int32_t k;
    asm("s_mov_b32 %0, %1" : "=s"(k) : "i"(CF));
    return k;
  }
}

// x * c for a compile-time coefficient.  S24: the caller proved |x| < 2^23, so
// the full-rate 24-bit multiplier gives the exact product.
template <int64_t CF, bool S24>
__device__ __forceinline__ int32_t mulc(int32_t x) {
  constexpr int64_t a = CF < 0 ? -CF : CF;
  if constexpr (CF == 1)
    return x;
  else if constexpr (CF == -1)
    return -x;
  else if constexpr ((a & (a - 1)) == 0)
    return x * (int32_t)CF;                      // shift
  else if constexpr (S24 && a < (1 << 23))
    return llvm_mul_i24(x, sconst<(int32_t)CF>());
  else
    return x * (int32_t)CF;
}
// acc + x * c in one instruction.  The compiler would split a multiply-add by
// a literal into v_mul_i32_i24 (literal form) plus an add; spelling the
// instruction out with the constant in a scalar register keeps it one op.
template <int64_t CF, bool S24>
__device__ __forceinline__ int32_t madc(int32_t x, int32_t acc) {
  constexpr int64_t a = CF < 0 ? -CF : CF;
  if constexpr (CF == 1) {
    return acc + x;
  } else if constexpr (CF == -1) {
    return acc - x;
  } else if constexpr ((a & (a - 1)) == 0) {
    return acc + x * (int32_t)CF;                // shift-add
  } else if constexpr (S24 && a < (1 << 23)) {
    int32_t r;
    if constexpr (CF >= -16 && CF <= 64)
      asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(x), "n"((int32_t)CF), "v"(acc));
    else
      asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"((int32_t)CF), "v"(acc));
    return r;
  } else {
    return acc + x * (int32_t)CF;
  }
}

// 32-bit operand, 64-bit product (one v_mad_i64_i32 when accumulated).
template <int64_t CF>
__device__ __forceinline__ int64_t mulc_wide(int32_t x) {
  static_assert(CF >= INT32_MIN && CF <= INT32_MAX);
  return (int64_t)x * (int64_t)(int32_t)CF;
}
template <int64_t CF>
__device__ __forceinline__ int64_t mulc_wide(int64_t x) {
  return x * CF;
}

constexpr bool coef_fit_i32(const IMat& t) {
  for (int i = 0; i < t.rows; ++i)
    for (int j = 0; j < t.cols; ++j)
      if (t.N[i][j] > INT32_MAX || t.N[i][j] < INT32_MIN) return false;
  return true;
}

// ---------------------------------------------------------------------------
// Arithmetic kinds.  Every value of a sandwich N x N^T is an integer with a
// compile-time bound; it is held in the cheapest type that is exact for it:
//   kI32  below 2^31: 32-bit integer multiply-adds;
//   kF64  below 2^53: a double.  Products and partial sums are integers below
//         2^53, so fp64 fused multiply-adds are exact, cost half a 64-bit
//         integer multiply-add, and the result converts to fp32 (round to
//         nearest even, what the cast needs) in one instruction;
//   kI64  the rest: 64-bit integers.
// The bound holds entry by entry: |(N x N^T)[i][j]| <= in_max |row i| |row j|
// (sums of absolute values) and |(N x)[i][b]| <= in_max |row i|, and so does
// every partial sum towards them.
// ---------------------------------------------------------------------------
enum { kI32 = 0, kF64 = 1, kI64 = 2 };
template <int KIND>
using kind_t = std::conditional_t<KIND == kI32, int32_t, std::conditional_t<KIND == kF64, double, int64_t>>;

template <const IMat& T, int64_t IN_MAX>
constexpr int raw_entry_kind(int i, int j) {
  const __int128 b = (__int128)IN_MAX * row_abs(T, i) * row_abs(T, j);
  return b < ((__int128)1 << 31) ? kI32 : b < ((__int128)1 << 53) ? kF64 : kI64;
}
// First pass, row i of N x.  A row that feeds a 64-bit entry stays integer (a
// double would have to be converted back); 32 bits need 32-bit coefficients.
template <const IMat& T, int64_t IN_MAX>
constexpr int tmp_kind(int i) {
  const __int128 b = (__int128)IN_MAX * row_abs(T, i);
  if (b < ((__int128)1 << 31) && coef_fit_i32(T)) return kI32;
  for (int j = 0; j < T.rows; ++j)
    if (raw_entry_kind<T, IN_MAX>(i, j) == kI64) return kI64;
  return b < ((__int128)1 << 53) ? kF64 : kI64;
}
// Second pass, entry (i, j): 32-bit arithmetic needs a 32-bit row i of N x.
template <const IMat& T, int64_t IN_MAX>
constexpr int entry_kind(int i, int j) {
  const int k = raw_entry_kind<T, IN_MAX>(i, j);
  return (k == kI32 && tmp_kind<T, IN_MAX>(i) != kI32) ? kF64 : k;
}
template <const IMat& T, int64_t IN_MAX>
constexpr bool all_tmp_i32() {
  for (int i = 0; i < T.rows; ++i)
    if (tmp_kind<T, IN_MAX>(i) != kI32) return false;
  return true;
}

// Storage: an array of int32_t where every value is kI32, else of 8-byte
// slots that hold an int32 (sign-extended), the bits of a double, or an int64.
template <typename Slot, typename V>
__device__ __forceinline__ Slot to_slot(V v) {
  if constexpr (sizeof(Slot) == 4)
    return (int32_t)v;
  else if constexpr (std::is_same_v<V, double>)
    return __builtin_bit_cast(int64_t, v);
  else
    return (int64_t)v;
}
template <int KIND, typename Slot>
__device__ __forceinline__ auto from_slot(Slot s) {
  if constexpr (sizeof(Slot) == 4 || KIND == kI64)
    return s;
  else if constexpr (KIND == kF64)
    return __builtin_bit_cast(double, s);
  else
    return (int32_t)s;
}
template <const IMat& T, int64_t IN_MAX>
using tmp_slot_t = std::conditional_t<all_tmp_i32<T, IN_MAX>(), int32_t, int64_t>;

// Rows of a Toom-Cook matrix built on points +p / -p come in pairs that agree
// on the even columns and differ by sign on the odd ones: row_j[a] =
// (-1)^a row_i[a].  Such a pair is evaluated as e + o and e - o from one even
// part and one odd part.  Returns the partner row of i, or -1.
constexpr int partner_of(const IMat& t, int i) {
  bool has_even = false, has_odd = false;
  for (int a = 0; a < t.cols; ++a)
    if (t.N[i][a] != 0) (a & 1 ? has_odd : has_even) = true;
  if (!has_even || !has_odd) return -1;
  for (int j = 0; j < t.rows; ++j) {
    if (j == i || t.rho[j] != t.rho[i]) continue;
    bool ok = true;
    for (int a = 0; a < t.cols; ++a)
      if (t.N[j][a] != ((a & 1) ? -t.N[i][a] : t.N[i][a])) ok = false;
    if (ok) return j;
  }
  return -1;
}

// Is column a the first non-zero of row i among the columns of parity PAR
// (0 even, 1 odd, 2 all)?
constexpr bool first_nz_par(const IMat& t, int i, int a, int par) {
  for (int k = 0; k < a; ++k)
    if (t.N[i][k] != 0 && (par == 2 || (k & 1) == par)) return false;
  return true;
}

// sum over the columns a of parity PAR of T.N[ROW][a] * get(a), accumulated in
// kind KIND; get(a) yields an int32_t, a double or an int64_t.
// S24: |get(a)| < 2^23 (32-bit kind only).
template <const IMat& T, int ROW, int PAR, bool S24, int KIND, class Get>
__device__ __forceinline__ kind_t<KIND> row_dot(Get&& get) {
  kind_t<KIND> acc = 0;
  static_for<0, T.cols>([&](auto a) {
    constexpr int A = decltype(a)::value;
    constexpr int64_t c = T.N[ROW][A];
    if constexpr (c != 0 && (PAR == 2 || (A & 1) == PAR)) {
      constexpr bool first = first_nz_par(T, ROW, A, PAR);
      const auto v = get(a);
      if constexpr (KIND == kI32) {
        if constexpr (first)
          acc = mulc<c, S24>((int32_t)v);
        else
          acc = madc<c, S24>((int32_t)v, acc);
      } else if constexpr (KIND == kF64) {
        if constexpr (first)
          acc = (double)v * (double)c;
        else
          acc = __builtin_fma((double)v, (double)c, acc);
      } else {
        static_assert(!std::is_same_v<std::decay_t<decltype(v)>, double>);
        acc += mulc_wide<c>(v);
      }
    }
  });
  return acc;
}

// One pass of a sandwich with |x| <= IN_MAX: out[i] = sum_a T.N[i][a] * get(a)
// for every row i, with paired rows sharing their even and odd parts (the rows
// of a pair have equal bounds, hence one kind).  put(i, value) receives the
// results.  LROW < 0: first pass, row i of N x, in tmp_kind(i).  LROW >= 0:
// second pass, entry (LROW, i) of N x N^T, in entry_kind(LROW, i).
template <const IMat& T, bool S24, int64_t IN_MAX, int LROW, class Get, class Put>
__device__ __forceinline__ void apply_rows(Get&& get, Put&& put) {
  static_for<0, T.rows>([&](auto i) {
    constexpr int I = decltype(i)::value;
    constexpr int PJ = partner_of(T, I);
    constexpr int KIND = LROW < 0 ? tmp_kind<T, IN_MAX>(I) : entry_kind<T, IN_MAX>(LROW < 0 ? 0 : LROW, I);
    if constexpr (PJ > I) {
      const auto e = row_dot<T, I, 0, S24, KIND>(get);
      const auto o = row_dot<T, I, 1, S24, KIND>(get);
      put(i, e + o);
      put(IC<PJ>{}, e - o);
    } else if constexpr (PJ < 0) {
      put(i, row_dot<T, I, 2, S24, KIND>(get));
    }
  });
}

// num = N x N^T with N the compile-time integer matrix T.N (T.rows x T.cols)
// and |x| <= IN_MAX.  Zero coefficients generate no code.  The entries of num
// are read back with entry<T, IN_MAX, I, J>().
template <const IMat& T, int64_t IN_MAX, typename AccT, typename InT>
__device__ __forceinline__ void sandwich(const InT (&x)[T.cols][T.cols],
                                         AccT (&num)[T.rows][T.rows]) {
  static_assert(std::is_same_v<AccT, acc_t<T, IN_MAX>>);
  constexpr bool s1 = IN_MAX < (1 << 23);
  constexpr bool s2 = (__int128)IN_MAX * T.rowsum < (1 << 23);
  using TmpT = tmp_slot_t<T, IN_MAX>;
  TmpT tmp[T.rows][T.cols];
  static_for<0, T.cols>([&](auto b) {                      // tmp = N x, column by column
    apply_rows<T, s1, IN_MAX, -1>([&](auto a) { return x[a][b]; },
                                  [&](auto i, auto v) { tmp[i][b] = to_slot<TmpT>(v); });
  });
  static_for<0, T.rows>([&](auto i) {                      // num = tmp N^T, row by row
    constexpr int I = decltype(i)::value;
    apply_rows<T, s2, IN_MAX, I>(
        [&](auto b) { return from_slot<tmp_kind<T, IN_MAX>(I)>(tmp[i][b]); },
        [&](auto j, auto v) { num[i][j] = to_slot<AccT>(v); });
  });
}

// The value of entry (I, J) of a sandwich result, in the type of its kind.
template <const IMat& T, int64_t IN_MAX, int I, int J, typename AccT>
__device__ __forceinline__ auto entry(AccT v) {
  return from_slot<entry_kind<T, IN_MAX>(I, J)>(v);
}

// ---------------------------------------------------------------------------
// Second bracket of a pair, fed with the 8-bit codes of the inner cast while they
// are still biased floats (cast_biased: 1.5 * 2^23 + q; the low half of the
// pattern is q as a 16-bit integer).  Where every coefficient of T.N fits 16 bits
// the first pass runs on v_dot2_i32_i16: the codes of two columns are packed into
// one register (one v_perm_b32 per pair, instead of one bias subtraction per
// code) and a dot product takes two coefficients at a time.  Columns are paired
// (0,2) (1,3) (4,6) (5,7) ..., so that a pair has one parity and serves the even /
// odd parts that paired rows share; a last pair (cols-2, cols-1) of mixed parity
// takes a zero coefficient for the column that is not wanted.  All sums are exact
// 32-bit integers as before.  Otherwise the bias is subtracted and sandwich() runs.
// ---------------------------------------------------------------------------
typedef short v2s __attribute__((ext_vector_type(2)));

template <const IMat& T, int64_t IN_MAX>
constexpr bool dot2_first_pass() {
  if (IN_MAX > 127 || !all_tmp_i32<T, IN_MAX>() || T.cols % 2 != 0) return false;
  for (int i = 0; i < T.rows; ++i)
    for (int a = 0; a < T.cols; ++a)
      if (T.N[i][a] > 32767 || T.N[i][a] < -32768) return false;
  return true;
}
// Columns of pair Q (see above).
constexpr int pair_col(int cols, int q, int which) {
  const int block = q / 2 * 4;
  if (block + 3 < cols) return block + (q & 1) + 2 * which;
  return cols - 2 + which;
}
// Coefficient of row ROW at column A if that column has parity PAR (2: any), else 0.
template <const IMat& T, int ROW, int PAR>
constexpr int64_t par_coef(int a) {
  return (PAR == 2 || (a & 1) == PAR) ? T.N[ROW][a] : 0;
}
// sum over the columns of parity PAR of T.N[ROW][a] * code[a], codes packed in pairs.
template <const IMat& T, int ROW, int PAR>
__device__ __forceinline__ int32_t row_dot2(const uint32_t (&pk)[T.cols / 2]) {
  int32_t acc = 0;
  static_for<0, T.cols / 2>([&](auto q) {
    constexpr int Q = decltype(q)::value;
    constexpr int64_t c0 = par_coef<T, ROW, PAR>(pair_col(T.cols, Q, 0));
    constexpr int64_t c1 = par_coef<T, ROW, PAR>(pair_col(T.cols, Q, 1));
    if constexpr (c0 != 0 || c1 != 0) {
      constexpr uint32_t k = (uint32_t)(uint16_t)(int16_t)c0 | ((uint32_t)(uint16_t)(int16_t)c1 << 16);
      // Saturation on: no sum here can reach 2^31 (all_tmp_i32), so it never acts; it selects
      // the three-operand form, whose accumulator may be the constant 0 (the two-operand
      // v_dot2c accumulates in place and would need a zeroed register per chain).
      acc = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, pk[Q]), __builtin_bit_cast(v2s, k), acc,
                                   true);
    }
  });
  return acc;
}

template <const IMat& T, int64_t IN_MAX, typename AccT>
__device__ __forceinline__ void sandwich_codes(const uint32_t (&bits)[T.cols][T.cols],
                                               AccT (&num)[T.rows][T.rows]) {
  static_assert(std::is_same_v<AccT, acc_t<T, IN_MAX>>);
  if constexpr (dot2_first_pass<T, IN_MAX>()) {
    constexpr bool s2 = (__int128)IN_MAX * T.rowsum < (1 << 23);
    int32_t tmp[T.rows][T.cols];
    static_for<0, T.cols>([&](auto b) {                    // tmp = N x, column by column
      uint32_t pk[T.cols / 2];
      static_for<0, T.cols / 2>([&](auto q) {
        constexpr int Q = decltype(q)::value;
        // low halves of the two patterns: (code of the first column) | (code of the second) << 16
        pk[Q] = __builtin_amdgcn_perm(bits[pair_col(T.cols, Q, 1)][b], bits[pair_col(T.cols, Q, 0)][b],
                                      0x05040100u);
      });
      static_for<0, T.rows>([&](auto i) {
        constexpr int I = decltype(i)::value;
        constexpr int PJ = partner_of(T, I);
        if constexpr (PJ > I) {
          const int32_t e = row_dot2<T, I, 0>(pk), o = row_dot2<T, I, 1>(pk);
          tmp[I][b] = e + o;
          tmp[PJ][b] = e - o;
        } else if constexpr (PJ < 0) {
          tmp[I][b] = row_dot2<T, I, 2>(pk);
        }
      });
    });
    static_for<0, T.rows>([&](auto i) {                    // num = tmp N^T, row by row
      constexpr int I = decltype(i)::value;
      apply_rows<T, s2, IN_MAX, I>([&](auto b) { return tmp[i][b]; },
                                   [&](auto j, auto v) { num[i][j] = to_slot<AccT>(v); });
    });
  } else {
    int x[T.cols][T.cols];
    static_for<0, T.cols>([&](auto a) {
      static_for<0, T.cols>([&](auto b) { x[a][b] = (int)bits[a][b] - 0x4B400000; });
    });
    sandwich<T, IN_MAX>(x, num);
  }
}

// Numerator -> fp32 for a dequantised output.  64-bit numerators go through
// their two halves (two conversions and one fma): not the correctly rounded
// conversion, but within 2 ulp, which an fp32 output tolerates; casts to integer
// codes keep the exact single-rounding conversion.
template <typename V>
__device__ __forceinline__ float to_float_approx(V v) {
  if constexpr (std::is_same_v<V, int64_t>) {
    // v = hi * 2^32 + lo with a SIGNED low half, so small |v| has hi = 0
    const int32_t lo = (int32_t)v;
    const int32_t hi = (int32_t)(v >> 32) + (int32_t)((uint32_t)lo >> 31);
    return __builtin_fmaf((float)hi, 4294967296.0f, (float)lo);
  } else {
    return (float)v;
  }
}

// One symmetric cast: q = clamp(rint(v * mult), +-qmax), where rint rounds the
// EXACT product of the two fp32 numbers to the nearest integer, ties to even.
// One fused multiply-add does it: v * mult + 1.5 * 2^23 is rounded once, to a
// float whose ulp is 1, so the integer sits in the low mantissa bits.  Products
// beyond +-2^22 leave that binade but stay on the right side of the clamp,
// which is applied to the biased float (a cast costs: convert, fma, med3).
constexpr float kMagic = 12582912.0f;   // 1.5 * 2^23, bit pattern 0x4B400000
__device__ __forceinline__ int cast_code(float v, float mult, float qmax) {
  float t = __builtin_fmaf(v, mult, kMagic);
  t = __builtin_amdgcn_fmed3f(t, kMagic - qmax, kMagic + qmax);
  return __float_as_int(t) - 0x4B400000;
}
// The same cast left in its biased float form 1.5 * 2^23 + q: the code sits, in two's
// complement, in the low bits of the returned pattern, so packing needs only its low byte
// (or half).
__device__ __forceinline__ uint32_t cast_biased(float v, float mult, float qmax) {
  float t = __builtin_fmaf(v, mult, kMagic);
  t = __builtin_amdgcn_fmed3f(t, kMagic - qmax, kMagic + qmax);
  return __float_as_uint(t);
}

// With one scale for the whole tensor the multiplier of entry (i, j) depends on the product
// rho_i rho_j of its row denominators only, so entries with equal products hold the same
// float: this is the index of the first of them (row-major).  Reading that one keeps a
// handful of multipliers in scalar registers instead of rows * rows (F(4,3) Legendre: 15
// for the base-change bracket, 3 for each main bracket, instead of 36 / 36 / 16).
template <const IMat& T, int I, int J>
constexpr int shared_mult_index() {
  for (int a = 0; a < T.rows; ++a)
    for (int b = 0; b < T.rows; ++b)
      if (T.rho[a] * T.rho[b] == T.rho[I] * T.rho[J]) return a * T.rows + b;
  return I * T.rows + J;
}

// Casts the result of sandwich<T, IN_MAX>, one multiplier per entry; entries
// that fit 32 bits are converted as such.  SHARE: the table was filled with one
// target scale (not per-point scales), see shared_mult_index.
template <const IMat& T, int64_t IN_MAX, bool SHARE = false, typename AccT>
__device__ __forceinline__ void cast_result(const AccT (&num)[T.rows][T.rows], const MultTable& mu,
                                            float qmax, int (&q)[T.rows][T.rows]) {
  static_for<0, T.rows>([&](auto i) {
    static_for<0, T.rows>([&](auto j) {
      constexpr int I = decltype(i)::value, J = decltype(j)::value;
      constexpr int at = SHARE ? shared_mult_index<T, I, J>() : I * T.rows + J;
      q[i][j] = cast_code((float)entry<T, IN_MAX, I, J>(num[i][j]), mu.v[at], qmax);
    });
  });
}

// The same casts left in their biased float form (for sandwich_codes).
template <const IMat& T, int64_t IN_MAX, bool SHARE = false, typename AccT>
__device__ __forceinline__ void cast_result_biased(const AccT (&num)[T.rows][T.rows],
                                                   const MultTable& mu, float qmax,
                                                   uint32_t (&q)[T.rows][T.rows]) {
  static_for<0, T.rows>([&](auto i) {
    static_for<0, T.rows>([&](auto j) {
      constexpr int I = decltype(i)::value, J = decltype(j)::value;
      constexpr int at = SHARE ? shared_mult_index<T, I, J>() : I * T.rows + J;
      q[i][j] = cast_biased((float)entry<T, IN_MAX, I, J>(num[i][j]), mu.v[at], qmax);
    });
  });
}

// ---------------------------------------------------------------------------
// Weight transform: one lane per (k, c) filter; a work group owns 256
// consecutive filters (K * C is a multiple of 256, so every block is full).
// Their 2304 input bytes are contiguous: 144 lanes fetch them with 16-byte
// loads into LDS and every lane picks its nine taps; the n*n results go back
// through LDS ([point][filter]) to 16-byte stores, as in the input transform.
// ---------------------------------------------------------------------------
template <int M, bool LEG, int BASE = 1>
__device__ __forceinline__ void weight_body(const int8_t* __restrict__ w, int8_t* __restrict__ V,
                                            const Geometry& g, const StageMults& mu,
                                            unsigned block) {
  constexpr int n = M + 2, n2 = n * n;
  using TB = Tab<M, BASE>;
  __shared__ __attribute__((aligned(16))) int8_t s_w[256 * 9];
  __shared__ __attribute__((aligned(16))) int8_t s_v[n2 * 256];
  const int tid = threadIdx.x;
  const long gid0 = (long)block * 256;
  const long KC = (long)g.K * g.C;
  // Fragment order: the block's 256 filters are 4 output channels x one 64-channel chunk
  // (item 64 r + j = filter (4 kq + r, 64 chunk + j)): their taps are 4 runs of up to 576
  // contiguous bytes, and a point's results are four 64-byte pieces of a fragment.  Filters
  // past C (partial last chunk) are dead: zero taps in, nothing stored.
  const int nch = (g.C + 63) >> 6;
  const int kq = g.frag ? (int)fast_div(block, g.mul_ch, g.sh_ch) : 0;
  const int chunk = g.frag ? (int)block - kq * nch : 0;
  const int cw = g.frag ? min(64, g.C - chunk * 64) : 64;      // channels of this chunk
  if (tid < 144) {
    const int8_t* src = w + gid0 * 9 + tid * 16;
    bool ok = true;
    if (g.frag) {
      const int run = tid / 36, piece = tid % 36;
      ok = piece * 16 < cw * 9;
      src = w + ((long)(kq * 4 + run) * g.C + chunk * 64) * 9 + piece * 16;
    }
    v4i v = {0, 0, 0, 0};
    if (ok) v = *reinterpret_cast<const v4i*>(src);
    *reinterpret_cast<v4i*>(s_w + tid * 16) = v;
  }
  __syncthreads();
  int wi[3][3];
  static_for<0, 3>([&](auto a) {
    static_for<0, 3>([&](auto b) { wi[a][b] = s_w[tid * 9 + decltype(a)::value * 3 + decltype(b)::value]; });
  });
  int q[n][n];
  if constexpr (LEG) {
    acc_t<TB::GP, 127> num1[n][n];
    sandwich<TB::GP, 127>(wi, num1);
    uint32_t w1[n][n];
    cast_result_biased<TB::GP, 127, true>(num1, mu.inner, 127.f, w1);
    acc_t<TB::Pinv, 127> num2[n][n];
    sandwich_codes<TB::Pinv, 127>(w1, num2);
    cast_result<TB::Pinv, 127>(num2, mu.outer, 127.f, q);
  } else {
    acc_t<TB::G, 127> num[n][n];
    sandwich<TB::G, 127>(wi, num);
    cast_result<TB::G, 127>(num, mu.outer, 127.f, q);
  }
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) {
      s_v[(decltype(i)::value * n + decltype(j)::value) * 256 + tid] = (int8_t)q[i][j];
    });
  });
  __syncthreads();
  int u = tid & 15;
  const int prow = tid >> 4;
  int8_t* vb = V + gid0 + u * 16;
  long pstride = KC;
  bool sok = true;
  if (g.frag) {
    // lane -> unit transposed, so that the four lanes of a quad store 64 contiguous bytes:
    // unit u = (filter row r = u / 4, 16-channel slice s = u % 4) of the block
    u = ((u & 3) << 2) | (u >> 2);
    const int r = u >> 2, sl = u & 3, k = kq * 4 + r;
    vb = V + ((long)(k >> 4) * nch + chunk) * 1024 + sl * 256 + (k & 15) * 16;
    pstride = ((long)(g.K + 15) >> 4) * nch * 1024;
    sok = sl * 16 < cw;
  }
#pragma unroll
  for (int it = 0; it < (n2 + 15) / 16; ++it) {
    const int p = it * 16 + prow;
    if (p < n2 && sok)
      __builtin_nontemporal_store(*reinterpret_cast<const v4i*>(s_v + p * 256 + u * 16),
                                  reinterpret_cast<v4i*>(vb + (long)p * pstride));
  }
}

// ---------------------------------------------------------------------------
// Input transform: one lane per (tile, channel).  A work group owns 256
// consecutive (tile, channel) items (channel fastest).  Because C is a
// multiple of 16, each 16-byte unit of that range lies inside one tile, so the
// block's input pixels are fetched with 16-byte loads into LDS ([pixel][item]),
// every lane then reads its own channel byte per pixel, and the n*n results go
// back through LDS ([point][item]) to 16-byte stores.  HBM and the texture
// path see only 16-byte accesses; the byte traffic stays inside LDS.
// Out-of-image pixels are staged as zeros.
// ---------------------------------------------------------------------------
// WHOLE: C is a multiple of 256, so the 256 items of a work group are 256
// channels of ONE tile: the tile index and everything derived from it is
// block-uniform (scalar registers, scalar arithmetic) and no item is out of
// range.
template <int M, bool LEG, bool WHOLE, int BASE = 1>
__device__ __forceinline__ void input_body(const int8_t* __restrict__ x, int8_t* __restrict__ U,
                                           const Geometry& g, const StageMults& mu,
                                           unsigned block) {
  constexpr int n = M + 2, n2 = n * n;
  using TB = Tab<M, BASE>;
  __shared__ __attribute__((aligned(16))) int8_t s_in[n2 * 256];
  __shared__ __attribute__((aligned(16))) int8_t s_out[n2 * 256];
  const int tid = threadIdx.x;
  const long gid0 = (long)block * 256;
  const long total = (long)g.T * g.C;

  // staging role of this lane: 16-byte unit `u` of the block's item range
  const int u = tid & 15, prow = tid >> 4;
  const long ug = gid0 + u * 16;
  int ut, uc;
  bool uok = WHOLE || ug < total;
  if constexpr (WHOLE) {
    ut = (int)fast_div(block, g.mul_cg, g.sh_cg);                    // uniform: C / 256 groups per tile
    uc = (int)(block - (unsigned)ut * (unsigned)(g.C >> 8)) * 256 + u * 16;
  } else if (g.frag) {
    // Fragment order: the block's 256 items are 4 tiles x one 64-channel chunk (unit u = tile
    // 4 tq + u / 4, channels 64 chunk + 16 (u % 4) ...): a quad of lanes loads 64 contiguous
    // bytes of a pixel, and a point's results are four 64-byte pieces of a fragment.
    const int nch = (g.C + 63) >> 6;
    const int quad = (int)fast_div(block, g.mul_ch, g.sh_ch);      // uniform
    ut = quad * 4 + (u >> 2);
    uc = ((int)block - quad * nch) * 64 + (u & 3) * 16;
    uok = ut < g.T && uc < g.C;
    if (!uok) ut = 0, uc = 0;
  } else {
    ut = uok ? (int)(ug / g.C) : 0;
    uc = uok ? (int)(ug - (long)ut * g.C) : 0;
  }
  int tx, ty, b;
  tile_coords(g, ut, b, ty, tx);
  const int8_t* xb = x + (long)b * g.H * g.W * g.C + uc;
  // Images of fewer than 2^23 pixels and 2^31 bytes (block-uniform): pixel offsets are
  // 32-bit, computed with the full-rate 24-bit multiplier (pixel index and C below 2^24,
  // product below 2^31), instead of 64-bit multiply-adds.
  const bool small_image = (long)g.H * g.W < (1L << 23) && (long)g.H * g.W * g.C < (1L << 31);
#pragma unroll
  for (int it = 0; it < (n2 + 15) / 16; ++it) {
    const int pix = it * 16 + prow;
    if (pix < n2) {
      const int a = pix / n, bb = pix - a * n;
      const int h = ty * M - 1 + a, ww = tx * M - 1 + bb;
      v4i v = {0, 0, 0, 0};
      if (uok && (unsigned)h < (unsigned)g.H && (unsigned)ww < (unsigned)g.W) {
        if constexpr (WHOLE)   // the launcher keeps H * W * C below 2^31 on this path
          v = *reinterpret_cast<const v4i*>(xb + (uint32_t)((h * g.W + ww) * g.C));
        else if (small_image)
          v = *reinterpret_cast<const v4i*>(xb + __umul24(__umul24(h, g.W) + ww, g.C));
        else
          v = *reinterpret_cast<const v4i*>(xb + ((long)h * g.W + ww) * g.C);
      }
      *reinterpret_cast<v4i*>(s_in + pix * 256 + u * 16) = v;
    }
  }
  __syncthreads();

  int xi[n][n];
  static_for<0, n>([&](auto a) {
    static_for<0, n>([&](auto bb) {
      xi[a][bb] = s_in[(decltype(a)::value * n + decltype(bb)::value) * 256 + tid];
    });
  });
  int q[n][n];
  if constexpr (LEG) {
    acc_t<TB::PinvT, 127> num1[n][n];
    sandwich<TB::PinvT, 127>(xi, num1);
    uint32_t x1[n][n];
    cast_result_biased<TB::PinvT, 127, true>(num1, mu.inner, 127.f, x1);
    acc_t<TB::BPT, 127> num2[n][n];
    sandwich_codes<TB::BPT, 127>(x1, num2);
    cast_result<TB::BPT, 127>(num2, mu.outer, 127.f, q);
  } else {
    acc_t<TB::BT, 127> num[n][n];
    sandwich<TB::BT, 127>(xi, num);
    cast_result<TB::BT, 127>(num, mu.outer, 127.f, q);
  }
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) {
      s_out[(decltype(i)::value * n + decltype(j)::value) * 256 + tid] = (int8_t)q[i][j];
    });
  });
  __syncthreads();

  int8_t* ub = U + (long)ut * g.C + uc;
  long pstride = total;
  int su = u;                                     // unit this lane stores
  bool sok = uok;
  if (g.frag) {
    // lane -> unit transposed, so that the four lanes of a quad store 64 contiguous bytes
    // (tiles 4 tq .. 4 tq + 3 of one 16-channel slice)
    su = ((u & 3) << 2) | (u >> 2);
    const int nch = (g.C + 63) >> 6;
    const int quad = (int)fast_div(block, g.mul_ch, g.sh_ch);
    const int st = quad * 4 + (su >> 2), sc = ((int)block - quad * nch) * 64 + (su & 3) * 16;
    sok = st < g.T && sc < g.C;
    ub = U + ((long)(st >> 4) * nch + (sc >> 6)) * 1024 + ((sc & 63) >> 4) * 256 + (st & 15) * 16;
    pstride = ((long)(g.T + 15) >> 4) * nch * 1024;
  }
#pragma unroll
  for (int it = 0; it < (n2 + 15) / 16; ++it) {
    const int p = it * 16 + prow;
    if (p < n2 && sok)
      __builtin_nontemporal_store(*reinterpret_cast<const v4i*>(s_out + p * 256 + su * 16),
                                  reinterpret_cast<v4i*>(ub + (long)p * pstride));
  }
}

template <int M, bool LEG, int BASE = 1>
__global__ __launch_bounds__(256) void k_weight_transform(const int8_t* __restrict__ w,
                                                          int8_t* __restrict__ V, Geometry g,
                                                          StageMults mu) {
  weight_body<M, LEG, BASE>(w, V, g, mu, blockIdx.x);
}

template <int M, bool LEG, bool WHOLE, int BASE = 1>
__global__ __launch_bounds__(256) void k_input_transform(const int8_t* __restrict__ x,
                                                         int8_t* __restrict__ U, Geometry g,
                                                         StageMults mu) {
  input_body<M, LEG, WHOLE, BASE>(x, U, g, mu, image_on_one_xcd(g, blockIdx.x));
}

// Both operand transforms in one launch (they are independent): one launch less per layer, and
// neither pays its own ramp-up and drain.  The first slots transform filters, the remaining
// `nb_in` ones input tiles.  Filters first, because their stores are the slow ones when the
// layer runs again and again: every L2 holds V's lines from the last contraction, and a line
// has to be dropped there before it can be written (measured on the 256-channel layer at
// N = 256: 24.1 -> 23.0 us per step against filters last).  The filter slots are padded to a
// multiple of 8, so that an input slot's XCD (slot % 8) is what image_on_one_xcd assumes.
template <int M, bool LEG, bool WHOLE, int BASE = 1>
__global__ __launch_bounds__(256) void k_operand_transforms(const int8_t* __restrict__ x,
                                                            int8_t* __restrict__ U,
                                                            const int8_t* __restrict__ w,
                                                            int8_t* __restrict__ V, Geometry g,
                                                            StageMults mu_in, StageMults mu_w,
                                                            unsigned nb_in) {
  const unsigned wslots = gridDim.x - nb_in;          // a multiple of 8
  if (blockIdx.x >= wslots)
    input_body<M, LEG, WHOLE, BASE>(x, U, g, mu_in, image_on_one_xcd(g, blockIdx.x - wslots));
  else if (blockIdx.x < weight_blocks(g))             // the padding slots have nothing to do
    weight_body<M, LEG, BASE>(w, V, g, mu_w, blockIdx.x);
}

// ---------------------------------------------------------------------------
// Output transform: one lane per (tile, output channel).
// OUT: 0 fp32 dequantised, 1 int32 numerators, 2 int8 codes.
// ---------------------------------------------------------------------------
template <typename MT>
struct MTraits;
template <>
struct MTraits<int8_t> {
  static constexpr int64_t in_max = 127;
};
template <>
struct MTraits<int16_t> {
  static constexpr int64_t in_max = 255;
};
template <>
struct MTraits<int32_t> {
  static constexpr int64_t in_max = kMaxAccUnquantised;
};

// WHOLE: K is a multiple of 256, so a work group's items are 256 output
// channels of ONE tile and the tile arithmetic is block-uniform.
// PP: M carries per-point power-of-two scales; the codes of point p enter the
// bracket shifted left by entry p of sh <= kMaxMShift, which the bounds account for.
template <int M, bool LEG, typename MT, int OUT, bool WHOLE, bool PP, int BASE = 1>
__global__ __launch_bounds__(256) void k_output_transform(const MT* __restrict__ Mq,
                                                          void* __restrict__ yv, Geometry g,
                                                          StageMults mu, int relu, ShiftTable sh) {
  constexpr int n = M + 2, n2 = n * n;
  constexpr int64_t IN_MAX = PP ? (MTraits<MT>::in_max << kMaxMShift) : MTraits<MT>::in_max;
  using TB = Tab<M, BASE>;
  const int tid = threadIdx.x;
  // WHOLE: the work groups of a run of tiles may be dealt to one XCD (the one whose
  // contraction blocks wrote those tiles' M)
  const unsigned block = WHOLE ? image_on_one_xcd(g, blockIdx.x) : blockIdx.x;
  const long gid0 = (long)block * 256;
  const long total = (long)g.T * g.K;
  const long gid = gid0 + tid;
  const bool active = WHOLE || gid < total;
  int t, k;
  if constexpr (WHOLE) {
    t = (int)fast_div(block, g.mul_kg, g.sh_kg);                     // uniform: K / 256 groups per tile
    k = (int)(block - (unsigned)t * (unsigned)(g.K >> 8)) * 256 + tid;
  } else {
    t = active ? (int)(gid / g.K) : 0;
    k = active ? (int)(gid - (long)t * g.K) : 0;
  }
  int tx, ty, b;
  tile_coords(g, t, b, ty, tx);

  int xi[n][n];
  if constexpr (sizeof(MT) == 1) {
    // int8 M: fetch the block's 256 consecutive (tile, k) items of every point
    // with 16-byte loads into LDS, then each lane picks its own byte.
    __shared__ __attribute__((aligned(16))) int8_t s_in[n2 * 256];
    const int u = tid & 15, prow = tid >> 4;
    const long ug = gid0 + u * 16;
    const bool uok = WHOLE || ug < total;
#pragma unroll
    for (int it = 0; it < (n2 + 15) / 16; ++it) {
      const int p = it * 16 + prow;
      if (p < n2) {
        v4i v = {0, 0, 0, 0};
        if (uok) v = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(Mq + (long)p * total + ug));
        *reinterpret_cast<v4i*>(s_in + p * 256 + u * 16) = v;
      }
    }
    __syncthreads();
    static_for<0, n>([&](auto i) {
      static_for<0, n>([&](auto j) {
        xi[i][j] = s_in[(decltype(i)::value * n + decltype(j)::value) * 256 + tid];
      });
    });
    if (!active) return;
  } else {
    if (!active) return;
    const MT* mb = Mq + (long)t * g.K + k;
    static_for<0, n>([&](auto i) {
      static_for<0, n>([&](auto j) {
        xi[i][j] = (int)__builtin_nontemporal_load(
            mb + (long)(decltype(i)::value * n + decltype(j)::value) * total);
      });
    });
  }

  if constexpr (PP) {
    static_for<0, n>([&](auto i) {
      static_for<0, n>([&](auto j) {
        xi[i][j] <<= sh.template at<decltype(i)::value * n + decltype(j)::value>();
      });
    });
  }

  // ReLU as a lower bound (none: below every value).  A float is bounded through its bit
  // pattern: negative values are negative integers, so one integer maximum with 0 clears
  // them (and -0.0), with INT_MIN it changes nothing.
  const int lo = relu ? 0 : (int)0x80000000;
  // Store addresses: with WHOLE the block is one tile, so everything but the lane's own
  // channel is block-uniform and stays in scalar registers; the lane's byte offset is made
  // opaque inside each store's block so that the sum is formed there and the store takes the
  // form scalar base + 32-bit lane offset (no vector address arithmetic).
  constexpr int YB = OUT == 2 ? 1 : 4;               // bytes of one output
  const long ytile = (((long)b * g.H + ty * M) * g.W + tx * M) * g.K;
  char* ybase = static_cast<char*>(yv) + (ytile + (WHOLE ? k - tid : k)) * YB;
  unsigned lane_off = WHOLE ? (unsigned)tid * YB : 0u;
  const int wk = g.W * g.K;
  auto finish = [&]<const IMat& FT, int64_t FIN>(auto& num) {
    static_for<0, M>([&](auto i) {
      static_for<0, M>([&](auto j) {
        // y has one scale: entries with equal row-denominator products share a multiplier
        constexpr int idx = shared_mult_index<FT, decltype(i)::value, decltype(j)::value>();
        const int h = ty * M + decltype(i)::value;
        const int ww = tx * M + decltype(j)::value;
        if (h < g.H && ww < g.W) {
          const int rel = decltype(i)::value * wk + decltype(j)::value * g.K;
          if constexpr (WHOLE) asm("" : "+v"(lane_off));
          char* at = ybase + (long)rel * YB + lane_off;
          if constexpr (OUT == 0) {
            float v = to_float_approx(entry<FT, FIN, decltype(i)::value, decltype(j)::value>(num[i][j])) * mu.outer.v[idx];
            __builtin_nontemporal_store(max(__float_as_int(v), lo), reinterpret_cast<int*>(at));
          } else if constexpr (OUT == 1) {
            int v = (int)entry<FT, FIN, decltype(i)::value, decltype(j)::value>(num[i][j]);
            __builtin_nontemporal_store(max(v, lo), reinterpret_cast<int*>(at));
          } else {
            int v = cast_code((float)entry<FT, FIN, decltype(i)::value, decltype(j)::value>(num[i][j]), mu.outer.v[idx], 127.f);
            __builtin_nontemporal_store((int8_t)max(v, lo), reinterpret_cast<int8_t*>(at));
          }
        }
      });
    });
  };
  if constexpr (LEG) {
    acc_t<TB::PinvT, IN_MAX> num1[n][n];
    sandwich<TB::PinvT, IN_MAX>(xi, num1);
    uint32_t m1[n][n];
    cast_result_biased<TB::PinvT, IN_MAX, true>(num1, mu.inner, 127.f, m1);
    acc_t<TB::APT, 127> num2[M][M];
    sandwich_codes<TB::APT, 127>(m1, num2);
    finish.template operator()<TB::APT, 127>(num2);
  } else {
    acc_t<TB::AT, IN_MAX> num[M][M];
    sandwich<TB::AT, IN_MAX>(xi, num);
    finish.template operator()<TB::AT, IN_MAX>(num);
  }
}

// ---------------------------------------------------------------------------
// Launchers of one M
// ---------------------------------------------------------------------------
template <int M>
hipError_t PerM<M>::weight(const Geometry& g, int br, const int8_t* w, int8_t* V,
                           const StageMults& mu, hipStream_t st) {
  const unsigned nb = weight_blocks(g);
  const bool leg = br != 0;
  if (br == 2)
    wino_launch((k_weight_transform<M, true, 2>), dim3(nb), dim3(256), st, w, V, g, mu);
  else if (br == 3)
    wino_launch((k_weight_transform<M, true, 3>), dim3(nb), dim3(256), st, w, V, g, mu);
  else if (leg)
    wino_launch((k_weight_transform<M, true>), dim3(nb), dim3(256), st, w, V, g, mu);
  else
    wino_launch((k_weight_transform<M, false>), dim3(nb), dim3(256), st, w, V, g, mu);
  return hipGetLastError();
}

template <int M>
hipError_t PerM<M>::input(const Geometry& g0, int br, const int8_t* x, int8_t* U,
                          const StageMults& mu, hipStream_t st) {
  const unsigned nb = input_blocks(g0);
  const bool whole = !g0.frag && whole_tiles(g0.C, g0.H, g0.W);
  const Geometry g = with_image_groups(g0, whole);
  const bool leg = br != 0;
  if (br == 2)
    wino_launch((k_input_transform<M, true, false, 2>), dim3(nb), dim3(256), st, x, U, g, mu);
  else if (br == 3)
    wino_launch((k_input_transform<M, true, false, 3>), dim3(nb), dim3(256), st, x, U, g, mu);
  else if (leg && whole)
    wino_launch((k_input_transform<M, true, true>), dim3(nb), dim3(256), st, x, U, g, mu);
  else if (leg)
    wino_launch((k_input_transform<M, true, false>), dim3(nb), dim3(256), st, x, U, g, mu);
  else if (whole)
    wino_launch((k_input_transform<M, false, true>), dim3(nb), dim3(256), st, x, U, g, mu);
  else
    wino_launch((k_input_transform<M, false, false>), dim3(nb), dim3(256), st, x, U, g, mu);
  return hipGetLastError();
}

template <int M>
hipError_t PerM<M>::operands(const Geometry& g0, int br, const int8_t* x, int8_t* U,
                             const int8_t* w, int8_t* V, const StageMults& mu_in,
                             const StageMults& mu_w, hipStream_t st) {
  const unsigned nb_in = input_blocks(g0), nb_w = weight_blocks(g0);
  const bool whole = !g0.frag && whole_tiles(g0.C, g0.H, g0.W);
  const Geometry g = with_image_groups(g0, whole);
  const dim3 grid(nb_in + (nb_w + 7) / 8 * 8), bs(256);   // filter slots padded to whole sets of XCDs
  const bool leg = br != 0;
  if (br == 2)
    wino_launch((k_operand_transforms<M, true, false, 2>), grid, bs, st, x, U, w, V, g, mu_in, mu_w, nb_in);
  else if (br == 3)
    wino_launch((k_operand_transforms<M, true, false, 3>), grid, bs, st, x, U, w, V, g, mu_in, mu_w, nb_in);
  else if (leg && whole)
    wino_launch((k_operand_transforms<M, true, true>), grid, bs, st, x, U, w, V, g, mu_in, mu_w, nb_in);
  else if (leg)
    wino_launch((k_operand_transforms<M, true, false>), grid, bs, st, x, U, w, V, g, mu_in, mu_w, nb_in);
  else if (whole)
    wino_launch((k_operand_transforms<M, false, true>), grid, bs, st, x, U, w, V, g, mu_in, mu_w, nb_in);
  else
    wino_launch((k_operand_transforms<M, false, false>), grid, bs, st, x, U, w, V, g, mu_in, mu_w, nb_in);
  return hipGetLastError();
}

template <int M, bool LEG, typename MT, bool WHOLE, bool PP>
static hipError_t output_mtw(const Geometry& g, const void* Mq, void* y, int out_type, bool relu,
                             const StageMults& mu, const ShiftTable& sh, hipStream_t st) {
  const dim3 nb(blocks_for((long)g.T * g.K)), bs(256);
  const MT* mp = static_cast<const MT*>(Mq);
  const int r = relu ? 1 : 0;
  if (out_type == 0) {
    wino_launch((k_output_transform<M, LEG, MT, 0, WHOLE, PP>), nb, bs, st, mp, y, g, mu, r, sh);
  } else if (out_type == 1) {
    // integer numerators only make sense for a single integer bracket with one scale
    if constexpr (LEG || PP)
      return hipErrorInvalidValue;
    else
      wino_launch((k_output_transform<M, LEG, MT, 1, WHOLE, PP>), nb, bs, st, mp, y, g, mu, r, sh);
  } else {
    wino_launch((k_output_transform<M, LEG, MT, 2, WHOLE, PP>), nb, bs, st, mp, y, g, mu, r, sh);
  }
  return hipGetLastError();
}

template <int M, bool LEG, typename MT>
static hipError_t output_mt(const Geometry& g, const void* Mq, void* y, int out_type, bool relu,
                            const StageMults& mu, const ShiftTable* sh, hipStream_t st) {
  if (sh) {
    if constexpr (sizeof(MT) == 4)
      return hipErrorInvalidValue;       // per-point scales need the 8- or 9-bit cast
    else
      return output_mtw<M, LEG, MT, false, true>(g, Mq, y, out_type, relu, mu, *sh, st);
  }
  const ShiftTable none{};
  // the block-uniform fast path is built for the int8 M of the all-8-bit pipeline
  if constexpr (sizeof(MT) == 1)
    if (whole_tiles(g.K, g.H, g.W))
      return output_mtw<M, LEG, MT, true, false>(with_output_groups(g), Mq, y, out_type, relu, mu, none, st);
  return output_mtw<M, LEG, MT, false, false>(g, Mq, y, out_type, relu, mu, none, st);
}

template <int M, bool LEG>
static hipError_t output_m(const Geometry& g, const void* Mq, int m_bits, void* y, int out_type,
                           bool relu, const StageMults& mu, const ShiftTable* sh, hipStream_t st) {
  if (m_bits == 8) return output_mt<M, LEG, int8_t>(g, Mq, y, out_type, relu, mu, sh, st);
  if (m_bits == 9) return output_mt<M, LEG, int16_t>(g, Mq, y, out_type, relu, mu, sh, st);
  return output_mt<M, LEG, int32_t>(g, Mq, y, out_type, relu, mu, sh, st);
}

// The Chebyshev and Hermite bases: the general kernel (per-lane tile arithmetic), per-tensor
// scales, fp32 or int8 output.
template <int M, int BASE>
static hipError_t output_base(const Geometry& g, const void* Mq, int m_bits, void* y, int out_type,
                              bool relu, const StageMults& mu, const ShiftTable* sh,
                              hipStream_t st) {
  if (sh || (out_type != 0 && out_type != 2)) return hipErrorInvalidValue;
  const dim3 nb(blocks_for((long)g.T * g.K)), bs(256);
  const ShiftTable none{};
  const int r = relu ? 1 : 0;
#define WINO_OUT_BASE(MT_)                                                                          \
  (out_type == 0                                                                                    \
       ? wino_launch((k_output_transform<M, true, MT_, 0, false, false, BASE>), nb, bs, st,         \
                     static_cast<const MT_*>(Mq), y, g, mu, r, none)                                \
       : wino_launch((k_output_transform<M, true, MT_, 2, false, false, BASE>), nb, bs, st,         \
                     static_cast<const MT_*>(Mq), y, g, mu, r, none))
  if (m_bits == 8)
    WINO_OUT_BASE(int8_t);
  else if (m_bits == 9)
    WINO_OUT_BASE(int16_t);
  else
    WINO_OUT_BASE(int32_t);
#undef WINO_OUT_BASE
  return hipGetLastError();
}

template <int M>
hipError_t PerM<M>::output(const Geometry& g, int br, const void* Mq, int m_bits, void* y,
                           int out_type, bool relu, const StageMults& mu, const ShiftTable* sh,
                           hipStream_t st) {
  if (br == 2) return output_base<M, 2>(g, Mq, m_bits, y, out_type, relu, mu, sh, st);
  if (br == 3) return output_base<M, 3>(g, Mq, m_bits, y, out_type, relu, mu, sh, st);
  return br ? output_m<M, true>(g, Mq, m_bits, y, out_type, relu, mu, sh, st)
            : output_m<M, false>(g, Mq, m_bits, y, out_type, relu, mu, sh, st);
}

}  // namespace wino
