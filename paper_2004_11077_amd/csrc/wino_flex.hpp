// "Flex" layer (Section 4.2): the brackets with G_P, B_P, A_P (G, B, A in the
// canonical base) use fp32 matrices supplied at run time -- trained parameters
// -- while the brackets with the fixed P^{-1} keep the exact integer arithmetic
// of the static kernels.  A run-time bracket T x T^T is evaluated on the
// integer codes in fp32 in one fixed order,
//     left[i][b] = ((T[i][0] x[0][b] + T[i][1] x[1][b]) + ...)
//     out[i][j]  = ((left[i][0] T[j][0] + left[i][1] T[j][1]) + ...)
// every product and every sum rounded to fp32, never fused, so that a CPU
// reference can follow it bit for bit; its cast uses one multiplier for the
// whole tensor.  These kernels serve trained matrices, whose entries have no
// structure to exploit: one lane per item, plain global accesses.
#pragma once
#include "wino_calibrate.hpp"

namespace wino {

// MODE of the kernels below
constexpr int kFlexRun = 0;       // produce the stage's tensor
constexpr int kFlexCalFloat = 1;  // amax[0] = max |value| of the fp32 bracket (float bits)
constexpr int kFlexCalInt = 2;    // weights, Legendre: per-(i,j) max |numerator| of the P^{-1} bracket

template <int ROWS, int COLS>
__device__ __forceinline__ void fsandwich(const float* __restrict__ Tm,
                                          const int (&x)[COLS][COLS], float (&out)[ROWS][ROWS]) {
#pragma clang fp contract(off)
  float left[ROWS][COLS];
  static_for<0, ROWS>([&](auto i) {
    static_for<0, COLS>([&](auto b) {
      float acc = Tm[decltype(i)::value * COLS] * (float)x[0][b];
      static_for<1, COLS>([&](auto a) {
        const float prod = Tm[decltype(i)::value * COLS + decltype(a)::value] * (float)x[a][b];
        acc = acc + prod;
      });
      left[i][b] = acc;
    });
  });
  static_for<0, ROWS>([&](auto i) {
    static_for<0, ROWS>([&](auto j) {
      float acc = left[i][0] * Tm[decltype(j)::value * COLS];
      static_for<1, COLS>([&](auto b) {
        const float prod = left[i][b] * Tm[decltype(j)::value * COLS + decltype(b)::value];
        acc = acc + prod;
      });
      out[i][j] = acc;
    });
  });
}

// Block-wide maximum of non-negative floats (as bit patterns), merged into amax[0].
__device__ __forceinline__ void merge_amax_float(float v, bool active,
                                                 unsigned long long* __restrict__ amax) {
  unsigned int u = active ? __float_as_uint(v) : 0u;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned int o = __shfl_xor(u, off);
    u = o > u ? o : u;
  }
  if ((threadIdx.x & 63) == 0 && u != 0) atomicMax(amax, (unsigned long long)u);
}

template <int R>
__device__ __forceinline__ float tile_absmax(const float (&v)[R][R]) {
  float best = 0.f;
  static_for<0, R>([&](auto i) {
    static_for<0, R>([&](auto j) { best = fmaxf(best, fabsf(v[i][j])); });
  });
  return best;
}

template <int M, bool LEG, int MODE>
__device__ __forceinline__ void flex_weight_body(const int8_t* __restrict__ w,
                                                 int8_t* __restrict__ V,
                                                 unsigned long long* __restrict__ amax,
                                                 const Geometry& g, const FlexMats& fm,
                                                 const StageMults& mu, float mult_first,
                                                 unsigned block) {
  constexpr int n = M + 2;
  using TB = Tab<M>;
  const long gid = (long)block * 256 + threadIdx.x;
  const long KC = (long)g.K * g.C;
  const bool active = gid < KC;
  int wi[3][3];
  static_for<0, 3>([&](auto a) {
    static_for<0, 3>([&](auto b) {
      wi[a][b] = active ? w[gid * 9 + decltype(a)::value * 3 + decltype(b)::value] : 0;
    });
  });
  float val[n][n];
  fsandwich<n, 3>(fm.GP, wi, val);
  if constexpr (MODE == kFlexCalFloat) {
    merge_amax_float(tile_absmax<n>(val), active, amax);
    return;
  }
  int q[n][n];
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) { q[i][j] = cast_code(val[i][j], mult_first, 127.f); });
  });
  if constexpr (LEG) {
    acc_t<TB::Pinv, 127> num2[n][n];
    sandwich<TB::Pinv, 127>(q, num2);
    if constexpr (MODE == kFlexCalInt) {
      merge_amax<TB::Pinv, 127>(num2, active, false, amax);
      return;
    }
    cast_result<TB::Pinv, 127>(num2, mu.outer, 127.f, q);
  }
  if (!active) return;
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) {
      V[(long)(decltype(i)::value * n + decltype(j)::value) * KC + gid] = (int8_t)q[i][j];
    });
  });
}

template <int M, bool LEG, int MODE>
__global__ __launch_bounds__(256) void k_flex_weight(const int8_t* __restrict__ w,
                                                     int8_t* __restrict__ V,
                                                     unsigned long long* __restrict__ amax,
                                                     Geometry g, FlexMats fm, StageMults mu,
                                                     float mult_first) {
  flex_weight_body<M, LEG, MODE>(w, V, amax, g, fm, mu, mult_first, blockIdx.x);
}

template <int M, bool LEG, int MODE>
__device__ __forceinline__ void flex_input_body(const int8_t* __restrict__ x,
                                                int8_t* __restrict__ U,
                                                unsigned long long* __restrict__ amax,
                                                const Geometry& g, const FlexMats& fm,
                                                const StageMults& mu, float mult_u,
                                                unsigned block) {
  constexpr int n = M + 2;
  using TB = Tab<M>;
  const long gid = (long)block * 256 + threadIdx.x;
  const long total = (long)g.T * g.C;
  const bool active = gid < total;
  const int t = active ? (int)(gid / g.C) : 0;
  const int c = active ? (int)(gid - (long)t * g.C) : 0;
  const int tx = t % g.TW;
  const int ty = (t / g.TW) % g.TH;
  const int b = t / (g.TW * g.TH);
  int xi[n][n];
  static_for<0, n>([&](auto a) {
    static_for<0, n>([&](auto bb) {
      const int h = ty * M - 1 + decltype(a)::value;
      const int ww = tx * M - 1 + decltype(bb)::value;
      int v = 0;
      if (active && h >= 0 && h < g.H && ww >= 0 && ww < g.W)
        v = x[(((long)b * g.H + h) * g.W + ww) * g.C + c];
      xi[a][bb] = v;
    });
  });
  if constexpr (LEG) {
    acc_t<TB::PinvT, 127> num1[n][n];
    sandwich<TB::PinvT, 127>(xi, num1);
    cast_result<TB::PinvT, 127>(num1, mu.inner, 127.f, xi);
  }
  float val[n][n];
  fsandwich<n, n>(fm.BPT, xi, val);
  if constexpr (MODE == kFlexCalFloat) {
    merge_amax_float(tile_absmax<n>(val), active, amax);
    return;
  }
  if (!active) return;
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) {
      U[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] =
          (int8_t)cast_code(val[i][j], mult_u, 127.f);
    });
  });
}

// OUT: 0 fp32 (mult_out = scale of the bracket's input), 2 int8 codes
// (mult_out = that scale / s_y).
template <int M, bool LEG, int MODE>
__global__ __launch_bounds__(256) void k_flex_input(const int8_t* __restrict__ x,
                                                    int8_t* __restrict__ U,
                                                    unsigned long long* __restrict__ amax,
                                                    Geometry g, FlexMats fm, StageMults mu,
                                                    float mult_u) {
  flex_input_body<M, LEG, MODE>(x, U, amax, g, fm, mu, mult_u, blockIdx.x);
}

// Both operand transforms of a layer in one launch (they are independent): the
// first nb_in work groups transform input tiles, the rest filters.
template <int M, bool LEG>
__global__ __launch_bounds__(256) void k_flex_operands(const int8_t* __restrict__ x,
                                                       int8_t* __restrict__ U,
                                                       const int8_t* __restrict__ w,
                                                       int8_t* __restrict__ V, Geometry g,
                                                       FlexMats fm, StageMults mu_in, float mult_u,
                                                       StageMults mu_w, float mult_first,
                                                       unsigned nb_in) {
  if (blockIdx.x < nb_in)
    flex_input_body<M, LEG, kFlexRun>(x, U, nullptr, g, fm, mu_in, mult_u, blockIdx.x);
  else
    flex_weight_body<M, LEG, kFlexRun>(w, V, nullptr, g, fm, mu_w, mult_first, blockIdx.x - nb_in);
}

template <int M, bool LEG, typename MT, int OUT, int MODE>
__global__ __launch_bounds__(256) void k_flex_output(const MT* __restrict__ Mq,
                                                     void* __restrict__ yv,
                                                     unsigned long long* __restrict__ amax,
                                                     Geometry g, FlexMats fm, StageMults mu,
                                                     float mult_out, int relu) {
  constexpr int n = M + 2;
  constexpr int64_t IN_MAX = MTraits<MT>::in_max;
  using TB = Tab<M>;
  const long total = (long)g.T * g.K;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const bool active = gid < total;
  const int t = active ? (int)(gid / g.K) : 0;
  const int k = active ? (int)(gid - (long)t * g.K) : 0;
  const int tx = t % g.TW;
  const int ty = (t / g.TW) % g.TH;
  const int b = t / (g.TW * g.TH);
  int xi[n][n];
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) {
      xi[i][j] = active ? (int)Mq[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] : 0;
    });
  });
  if constexpr (LEG) {
    acc_t<TB::PinvT, IN_MAX> num1[n][n];
    sandwich<TB::PinvT, IN_MAX>(xi, num1);
    cast_result<TB::PinvT, IN_MAX>(num1, mu.inner, 127.f, xi);
  }
  float val[M][M];
  fsandwich<M, n>(fm.APT, xi, val);
  if constexpr (MODE == kFlexCalFloat) {
    // positions cropped from partial tiles do not count; with relu only the
    // positive part has to be covered
    float best = 0.f;
    static_for<0, M>([&](auto i) {
      static_for<0, M>([&](auto j) {
        const bool inside = ty * M + decltype(i)::value < g.H && tx * M + decltype(j)::value < g.W;
        const float v = relu ? fmaxf(val[i][j], 0.f) : fabsf(val[i][j]);
        best = fmaxf(best, inside ? v : 0.f);
      });
    });
    merge_amax_float(best, active, amax);
    return;
  }
  if (!active) return;
  const long ybase = (((long)b * g.H + ty * M) * g.W + tx * M) * g.K + k;
  const int wk = g.W * g.K;
  static_for<0, M>([&](auto i) {
    static_for<0, M>([&](auto j) {
      const int h = ty * M + decltype(i)::value;
      const int ww = tx * M + decltype(j)::value;
      if (h < g.H && ww < g.W) {
        const int rel = decltype(i)::value * wk + decltype(j)::value * g.K;
        if constexpr (OUT == 0) {
          const float v = val[i][j] * mult_out;
          (static_cast<float*>(yv) + ybase)[rel] = relu ? fmaxf(v, 0.f) : v;
        } else {
          const int v = cast_code(val[i][j], mult_out, 127.f);
          (static_cast<int8_t*>(yv) + ybase)[rel] = (int8_t)(relu ? max(v, 0) : v);
        }
      }
    });
  });
}

template <int M>
hipError_t PerMFlex<M>::weight(const Geometry& g, bool leg, int mode, const int8_t* w, int8_t* V,
                               unsigned long long* amax, const FlexMats& fm,
                               const StageMults& mu, float mult_first, hipStream_t st) {
  const dim3 nb(blocks_for((long)g.K * g.C)), bs(256);
#define WINO_FLEX_W(LEG_, MODE_) \
  wino_launch((k_flex_weight<M, LEG_, MODE_>), nb, bs, st, w, V, amax, g, fm, mu, mult_first)
  if (mode == kFlexRun) {
    if (leg) WINO_FLEX_W(true, kFlexRun); else WINO_FLEX_W(false, kFlexRun);
  } else if (mode == kFlexCalFloat) {
    if (leg) WINO_FLEX_W(true, kFlexCalFloat); else WINO_FLEX_W(false, kFlexCalFloat);
  } else {
    if (!leg) return hipErrorInvalidValue;
    WINO_FLEX_W(true, kFlexCalInt);
  }
#undef WINO_FLEX_W
  return hipGetLastError();
}

template <int M>
hipError_t PerMFlex<M>::input(const Geometry& g, bool leg, int mode, const int8_t* x, int8_t* U,
                              unsigned long long* amax, const FlexMats& fm, const StageMults& mu,
                              float mult_u, hipStream_t st) {
  const dim3 nb(blocks_for((long)g.T * g.C)), bs(256);
#define WINO_FLEX_I(LEG_, MODE_) \
  wino_launch((k_flex_input<M, LEG_, MODE_>), nb, bs, st, x, U, amax, g, fm, mu, mult_u)
  if (mode == kFlexRun) {
    if (leg) WINO_FLEX_I(true, kFlexRun); else WINO_FLEX_I(false, kFlexRun);
  } else {
    if (leg) WINO_FLEX_I(true, kFlexCalFloat); else WINO_FLEX_I(false, kFlexCalFloat);
  }
#undef WINO_FLEX_I
  return hipGetLastError();
}

template <int M>
hipError_t PerMFlex<M>::operands(const Geometry& g, bool leg, const int8_t* x, int8_t* U,
                                 const int8_t* w, int8_t* V, const FlexMats& fm,
                                 const StageMults& mu_in, float mult_u, const StageMults& mu_w,
                                 float mult_first, hipStream_t st) {
  const unsigned nb_in = blocks_for((long)g.T * g.C), nb_w = blocks_for((long)g.K * g.C);
  const dim3 grid(nb_in + nb_w), bs(256);
  if (leg)
    wino_launch((k_flex_operands<M, true>), grid, bs, st, x, U, w, V, g, fm, mu_in, mult_u, mu_w,
                mult_first, nb_in);
  else
    wino_launch((k_flex_operands<M, false>), grid, bs, st, x, U, w, V, g, fm, mu_in, mult_u, mu_w,
                mult_first, nb_in);
  return hipGetLastError();
}

template <int M, bool LEG, typename MT>
static hipError_t flex_output_mt(const Geometry& g, int mode, const void* Mq, void* y,
                                 int out_type, bool relu, unsigned long long* amax,
                                 const FlexMats& fm, const StageMults& mu, float mult_out,
                                 hipStream_t st) {
  const dim3 nb(blocks_for((long)g.T * g.K)), bs(256);
  const MT* mp = static_cast<const MT*>(Mq);
  const int r = relu ? 1 : 0;
  if (mode == kFlexCalFloat)
    wino_launch((k_flex_output<M, LEG, MT, 0, kFlexCalFloat>), nb, bs, st, mp, y, amax, g, fm, mu,
                mult_out, r);
  else if (out_type == 0)
    wino_launch((k_flex_output<M, LEG, MT, 0, kFlexRun>), nb, bs, st, mp, y, amax, g, fm, mu,
                mult_out, r);
  else
    wino_launch((k_flex_output<M, LEG, MT, 2, kFlexRun>), nb, bs, st, mp, y, amax, g, fm, mu,
                mult_out, r);
  return hipGetLastError();
}

template <int M>
hipError_t PerMFlex<M>::output(const Geometry& g, bool leg, int mode, const void* Mq, int m_bits,
                               void* y, int out_type, bool relu, unsigned long long* amax,
                               const FlexMats& fm, const StageMults& mu, float mult_out,
                               hipStream_t st) {
#define WINO_FLEX_O(LEG_)                                                                        \
  (m_bits == 8   ? flex_output_mt<M, LEG_, int8_t>(g, mode, Mq, y, out_type, relu, amax, fm, mu, \
                                                   mult_out, st)                                 \
   : m_bits == 9 ? flex_output_mt<M, LEG_, int16_t>(g, mode, Mq, y, out_type, relu, amax, fm,    \
                                                    mu, mult_out, st)                            \
                 : flex_output_mt<M, LEG_, int32_t>(g, mode, Mq, y, out_type, relu, amax, fm,    \
                                                    mu, mult_out, st))
  return leg ? WINO_FLEX_O(true) : WINO_FLEX_O(false);
#undef WINO_FLEX_O
}

}  // namespace wino
