// fp32 brackets with the fixed rational matrices of eq. 1-4: T x T^T and its
// adjoint T^T x T, coefficients rounded to fp32 at compile time, zero
// coefficients generating no code, explicit fused multiply-adds.  Used by the
// fp32 forward path and by both backward passes.
#pragma once
#include <type_traits>

#include "wino_tables.hpp"

namespace wino {

template <int B, int E, class F>
__device__ __forceinline__ void rfor(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    rfor<B + 1, E>(f);
  }
}

// The rational matrices of F(M x M, 3 x 3) as template arguments.
template <int M>
struct TabF {
  static constexpr MatrixSet ms = standard_matrix_set(M);
  static constexpr RMat G = ms.G, BT = ms.BT, AT = ms.AT, PinvT = ms.PinvT, Pinv = ms.Pinv,
                        GP = ms.GP, BPT = ms.BPT, APT = ms.APT;
};

template <const RMat& T, int I, int J>
inline constexpr float kCoef = (float)((double)T.a[I][J].num / (double)T.a[I][J].den);

template <const RMat& T, int I, int J>
inline constexpr double kCoefD = (double)T.a[I][J].num / (double)T.a[I][J].den;

// out = T x T^T  (x: T.cols x T.cols, out: T.rows x T.rows).
template <const RMat& T>
__device__ __forceinline__ void bracket_f(const float (&x)[T.cols][T.cols],
                                          float (&out)[T.rows][T.rows]) {
  float tmp[T.rows][T.cols];
  rfor<0, T.rows>([&](auto i) {
    rfor<0, T.cols>([&](auto b) {
      float acc = 0.f;
      rfor<0, T.cols>([&](auto a) {
        constexpr int I = decltype(i)::value, A = decltype(a)::value;
        if constexpr (T.a[I][A].num != 0) acc = __builtin_fmaf(kCoef<T, I, A>, x[a][b], acc);
      });
      tmp[i][b] = acc;
    });
  });
  rfor<0, T.rows>([&](auto i) {
    rfor<0, T.rows>([&](auto j) {
      float acc = 0.f;
      rfor<0, T.cols>([&](auto b) {
        constexpr int J = decltype(j)::value, Bc = decltype(b)::value;
        if constexpr (T.a[J][Bc].num != 0) acc = __builtin_fmaf(kCoef<T, J, Bc>, tmp[i][b], acc);
      });
      out[i][j] = acc;
    });
  });
}

// The same bracket evaluated in double (coefficients rounded to double).  The
// two brackets of eq. 2 / eq. 4 multiply out to the canonical matrix, but each
// on its own has large entries of mixed sign (row sums of |B_P^T| near 100 for
// F(6,3)), so a bracket pair chained in fp32 loses the digits that cancel; the
// fp32 path therefore keeps the value between the two brackets, and their
// arithmetic, in double and rounds to fp32 only what it stores.
template <const RMat& T, typename In, typename Out>
__device__ __forceinline__ void bracket_d(const In (&x)[T.cols][T.cols],
                                          Out (&out)[T.rows][T.rows]) {
  double tmp[T.rows][T.cols];
  rfor<0, T.rows>([&](auto i) {
    rfor<0, T.cols>([&](auto b) {
      double acc = 0.0;
      rfor<0, T.cols>([&](auto a) {
        constexpr int I = decltype(i)::value, A = decltype(a)::value;
        if constexpr (T.a[I][A].num != 0) acc = __builtin_fma(kCoefD<T, I, A>, (double)x[a][b], acc);
      });
      tmp[i][b] = acc;
    });
  });
  rfor<0, T.rows>([&](auto i) {
    rfor<0, T.rows>([&](auto j) {
      double acc = 0.0;
      rfor<0, T.cols>([&](auto b) {
        constexpr int J = decltype(j)::value, Bc = decltype(b)::value;
        if constexpr (T.a[J][Bc].num != 0) acc = __builtin_fma(kCoefD<T, J, Bc>, tmp[i][b], acc);
      });
      out[i][j] = (Out)acc;
    });
  });
}

// out = T^T x T  (x: T.rows x T.rows, out: T.cols x T.cols): the adjoint of x -> T x T^T.
template <const RMat& T>
__device__ __forceinline__ void adjoint_bracket_f(const float (&x)[T.rows][T.rows],
                                                  float (&out)[T.cols][T.cols]) {
  float tmp[T.cols][T.rows];
  rfor<0, T.cols>([&](auto i) {
    rfor<0, T.rows>([&](auto b) {
      float acc = 0.f;
      rfor<0, T.rows>([&](auto a) {
        constexpr int I = decltype(i)::value, A = decltype(a)::value;
        if constexpr (T.a[A][I].num != 0) acc = __builtin_fmaf(kCoef<T, A, I>, x[a][b], acc);
      });
      tmp[i][b] = acc;
    });
  });
  rfor<0, T.cols>([&](auto i) {
    rfor<0, T.cols>([&](auto j) {
      float acc = 0.f;
      rfor<0, T.rows>([&](auto b) {
        constexpr int J = decltype(j)::value, Bc = decltype(b)::value;
        if constexpr (T.a[Bc][J].num != 0) acc = __builtin_fmaf(kCoef<T, Bc, J>, tmp[i][b], acc);
      });
      out[i][j] = acc;
    });
  });
}

// dV [n*n][K*C] may arrive as `parts` partial sums over ranges of tiles, n*n * total floats
// apart.  The one lane that reads filter gid adds them in ascending order and leaves the
// sums in the first part.  The first part is loaded whole; the others two rows of the
// N x N points at a time (2 N independent loads per step, kept apart so that the lane
// needs no second N x N array of registers: the kernels that call this share their
// register budget with a bandwidth-bound body that wants many waves).
template <int N>
__device__ __forceinline__ void load_summed_dv(float* __restrict__ dV, long total, long gid,
                                               int parts, bool active, float (&v)[N][N]) {
  static_assert(N % 2 == 0, "rows are taken in pairs");
  rfor<0, N>([&](auto i) {
    rfor<0, N>([&](auto j) {
      v[i][j] = active ? dV[(long)(decltype(i)::value * N + decltype(j)::value) * total + gid] : 0.f;
    });
  });
  if (parts <= 1 || !active) return;
  for (int sp = 1; sp < parts; ++sp) {
    const float* part = dV + (long)sp * N * N * total;
    rfor<0, N / 2>([&](auto ii) {
      constexpr int i0 = 2 * decltype(ii)::value;
      float t[2][N];
      rfor<0, 2>([&](auto d) {
        rfor<0, N>([&](auto j) {
          t[d][j] = part[(long)((i0 + decltype(d)::value) * N + decltype(j)::value) * total + gid];
        });
      });
      rfor<0, 2>([&](auto d) {
        rfor<0, N>([&](auto j) { v[i0 + decltype(d)::value][j] += t[d][j]; });
      });
      __builtin_amdgcn_sched_barrier(0);
    });
  }
  rfor<0, N>([&](auto i) {
    rfor<0, N>([&](auto j) {
      dV[(long)(decltype(i)::value * N + decltype(j)::value) * total + gid] = v[i][j];
    });
  });
}

}  // namespace wino
