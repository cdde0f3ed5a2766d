// Calibration kernels: per-(i, j) maxima of the integer numerators of one
// bracket, from which the host derives the per-tensor scale of that cast
// (scale = max |real| / qmax, real = num * s_prev / (rho_i rho_j)).  They reuse
// the exact integer sandwiches and casts of the transform kernels; they are
// run once per layer when its scales are chosen, so they are written for
// clarity, not speed (one lane per item, plain global loads).
#pragma once
#include "wino_transforms.hpp"

namespace wino {

// Block-wide maximum of |v| for each of the R*R entries of a result of
// sandwich<T, IN_MAX>, merged into amax[] (global).
template <const IMat& T, int64_t IN_MAX, typename AccT>
__device__ __forceinline__ void merge_amax(const AccT (&num)[T.rows][T.rows], bool active,
                                           bool positive_only,
                                           unsigned long long* __restrict__ amax) {
  __shared__ unsigned long long s_max[kMaxPts];
  if (threadIdx.x < kMaxPts) s_max[threadIdx.x] = 0;
  __syncthreads();
  constexpr int R = T.rows;
  static_for<0, R>([&](auto i) {
    static_for<0, R>([&](auto j) {
      long long v = (long long)entry<T, IN_MAX, decltype(i)::value, decltype(j)::value>(num[i][j]);
      if (positive_only)
        v = v > 0 ? v : 0;
      else
        v = v < 0 ? -v : v;
      unsigned long long u = active ? (unsigned long long)v : 0ull;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(u, off);
        u = o > u ? o : u;
      }
      if ((threadIdx.x & 63) == 0) atomicMax(&s_max[decltype(i)::value * R + decltype(j)::value], u);
    });
  });
  __syncthreads();
  if (threadIdx.x < R * R && s_max[threadIdx.x] != 0) atomicMax(&amax[threadIdx.x], s_max[threadIdx.x]);
}

// PHASE 1: numerators of the inner bracket (Legendre only).
// PHASE 2: numerators of the outer bracket (after the inner cast, if any).
template <int M, bool LEG, int PHASE>
__global__ __launch_bounds__(256) void k_cal_weight(const int8_t* __restrict__ w,
                                                    unsigned long long* __restrict__ amax,
                                                    Geometry g, StageMults mu) {
  constexpr int n = M + 2;
  using TB = Tab<M>;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const long KC = (long)g.K * g.C;
  const bool active = gid < KC;
  int wi[3][3];
  static_for<0, 3>([&](auto a) {
    static_for<0, 3>([&](auto b) {
      wi[a][b] = active ? w[gid * 9 + decltype(a)::value * 3 + decltype(b)::value] : 0;
    });
  });
  if constexpr (LEG) {
    acc_t<TB::GP, 127> num1[n][n];
    sandwich<TB::GP, 127>(wi, num1);
    if constexpr (PHASE == 1) {
      merge_amax<TB::GP, 127>(num1, active, false, amax);
    } else {
      int w1[n][n];
      cast_result<TB::GP, 127>(num1, mu.inner, 127.f, w1);
      acc_t<TB::Pinv, 127> num2[n][n];
      sandwich<TB::Pinv, 127>(w1, num2);
      merge_amax<TB::Pinv, 127>(num2, active, false, amax);
    }
  } else {
    acc_t<TB::G, 127> num[n][n];
    sandwich<TB::G, 127>(wi, num);
    merge_amax<TB::G, 127>(num, active, false, amax);
  }
}

template <int M, bool LEG, int PHASE>
__global__ __launch_bounds__(256) void k_cal_input(const int8_t* __restrict__ x,
                                                   unsigned long long* __restrict__ amax,
                                                   Geometry g, StageMults mu) {
  constexpr int n = M + 2;
  using TB = Tab<M>;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const bool active = gid < (long)g.T * g.C;
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
    if constexpr (PHASE == 1) {
      merge_amax<TB::PinvT, 127>(num1, active, false, amax);
    } else {
      int x1[n][n];
      cast_result<TB::PinvT, 127>(num1, mu.inner, 127.f, x1);
      acc_t<TB::BPT, 127> num2[n][n];
      sandwich<TB::BPT, 127>(x1, num2);
      merge_amax<TB::BPT, 127>(num2, active, false, amax);
    }
  } else {
    acc_t<TB::BT, 127> num[n][n];
    sandwich<TB::BT, 127>(xi, num);
    merge_amax<TB::BT, 127>(num, active, false, amax);
  }
}

// With relu the output scale only has to cover the positive numerators.
template <int M, bool LEG, typename MT, int PHASE, bool PP>
__global__ __launch_bounds__(256) void k_cal_output(const MT* __restrict__ Mq,
                                                    unsigned long long* __restrict__ amax,
                                                    Geometry g, StageMults mu, int relu,
                                                    ShiftTable sh) {
  constexpr int n = M + 2;
  constexpr int64_t IN_MAX = PP ? (MTraits<MT>::in_max << kMaxMShift) : MTraits<MT>::in_max;
  using TB = Tab<M>;
  const long total = (long)g.T * g.K;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const bool active = gid < total;
  int xi[n][n];
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) {
      xi[i][j] = active ? (int)Mq[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] : 0;
      if constexpr (PP) xi[i][j] <<= sh.template at<decltype(i)::value * n + decltype(j)::value>();
    });
  });
  // entries of partial tiles that fall outside the image are cropped, so they
  // must not count: mask them per output position
  const int t = active ? (int)(gid / g.K) : 0;
  const int tx = t % g.TW;
  const int ty = (t / g.TW) % g.TH;
  auto crop = [&](auto& num) {
    static_for<0, M>([&](auto i) {
      static_for<0, M>([&](auto j) {
        if (ty * M + decltype(i)::value >= g.H || tx * M + decltype(j)::value >= g.W) num[i][j] = 0;
      });
    });
  };
  if constexpr (LEG) {
    acc_t<TB::PinvT, IN_MAX> num1[n][n];
    sandwich<TB::PinvT, IN_MAX>(xi, num1);
    if constexpr (PHASE == 1) {
      merge_amax<TB::PinvT, IN_MAX>(num1, active, false, amax);
    } else {
      int m1[n][n];
      cast_result<TB::PinvT, IN_MAX>(num1, mu.inner, 127.f, m1);
      acc_t<TB::APT, 127> num2[M][M];
      sandwich<TB::APT, 127>(m1, num2);
      crop(num2);
      merge_amax<TB::APT, 127>(num2, active, relu != 0, amax);
    }
  } else {
    acc_t<TB::AT, IN_MAX> num[M][M];
    sandwich<TB::AT, IN_MAX>(xi, num);
    crop(num);
    merge_amax<TB::AT, IN_MAX>(num, active, relu != 0, amax);
  }
}

template <int M>
hipError_t PerMCal<M>::weight(const Geometry& g, bool leg, int phase, const int8_t* w,
                              unsigned long long* amax, const StageMults& mu, hipStream_t st) {
  const unsigned nb = (unsigned)(((long)g.K * g.C + 255) / 256);
  if (!leg)
    wino_launch((k_cal_weight<M, false, 2>), dim3(nb), dim3(256), st, w, amax, g, mu);
  else if (phase == 1)
    wino_launch((k_cal_weight<M, true, 1>), dim3(nb), dim3(256), st, w, amax, g, mu);
  else
    wino_launch((k_cal_weight<M, true, 2>), dim3(nb), dim3(256), st, w, amax, g, mu);
  return hipGetLastError();
}

template <int M>
hipError_t PerMCal<M>::input(const Geometry& g, bool leg, int phase, const int8_t* x,
                             unsigned long long* amax, const StageMults& mu, hipStream_t st) {
  const unsigned nb = (unsigned)(((long)g.T * g.C + 255) / 256);
  if (!leg)
    wino_launch((k_cal_input<M, false, 2>), dim3(nb), dim3(256), st, x, amax, g, mu);
  else if (phase == 1)
    wino_launch((k_cal_input<M, true, 1>), dim3(nb), dim3(256), st, x, amax, g, mu);
  else
    wino_launch((k_cal_input<M, true, 2>), dim3(nb), dim3(256), st, x, amax, g, mu);
  return hipGetLastError();
}

template <int M, typename MT, bool PP>
static hipError_t cal_output_mt(const Geometry& g, bool leg, int phase, const void* Mq,
                                unsigned long long* amax, const StageMults& mu, bool relu,
                                const ShiftTable& sh, hipStream_t st) {
  const dim3 nb((unsigned)(((long)g.T * g.K + 255) / 256)), bs(256);
  const MT* mp = static_cast<const MT*>(Mq);
  const int r = relu ? 1 : 0;
  if (!leg)
    wino_launch((k_cal_output<M, false, MT, 2, PP>), nb, bs, st, mp, amax, g, mu, r, sh);
  else if (phase == 1)
    wino_launch((k_cal_output<M, true, MT, 1, PP>), nb, bs, st, mp, amax, g, mu, r, sh);
  else
    wino_launch((k_cal_output<M, true, MT, 2, PP>), nb, bs, st, mp, amax, g, mu, r, sh);
  return hipGetLastError();
}

template <int M>
hipError_t PerMCal<M>::output(const Geometry& g, bool leg, int phase, const void* Mq, int m_bits,
                              unsigned long long* amax, const StageMults& mu, bool relu,
                              const ShiftTable* sh, hipStream_t st) {
  if (sh) {
    if (m_bits == 8) return cal_output_mt<M, int8_t, true>(g, leg, phase, Mq, amax, mu, relu, *sh, st);
    if (m_bits == 9) return cal_output_mt<M, int16_t, true>(g, leg, phase, Mq, amax, mu, relu, *sh, st);
    return hipErrorInvalidValue;
  }
  const ShiftTable none{};
  if (m_bits == 8) return cal_output_mt<M, int8_t, false>(g, leg, phase, Mq, amax, mu, relu, none, st);
  if (m_bits == 9) return cal_output_mt<M, int16_t, false>(g, leg, phase, Mq, amax, mu, relu, none, st);
  return cal_output_mt<M, int32_t, false>(g, leg, phase, Mq, amax, mu, relu, none, st);
}

}  // namespace wino
