// Backward pass of the flex layer (Section 4.2: G_P, B_P, A_P are trained, P and
// P^{-1} stay fixed), fp32, casts passing their gradient on unchanged.
// For a bracket R = T S T^T with a trained matrix T:
//     dT = sum over items of  dR (T S^T) + dR^T (T S),      dS = T^T dR T,
// and through a fixed bracket S1 = L S L^T:  dS = L^T dS1 L.  The inputs S of the
// trained brackets are recomputed from the forward pass's integer tensors with the
// forward pass's exact arithmetic (X1 from x, M1 from M) and dequantised.
//
//   k_fbwd_output   dY, M  -> dM, per-block partial sums of dA_P^T
//   fbwd_input_body   dU, x  -> per-tile dX, per-block partial sums of dB_P^T   \ one launch,
//   fbwd_weight_body  dV, w  -> dw, per-block partial sums of dG_P              / k_fbwd_input_weight
//   k_bwd_tile_sum  per-tile dX -> dx (fixed order over the <= 4 covering tiles)
//   k_sum_partials  partial sums -> the three matrix gradients (fixed order)
// The two contraction gradients between them are those of the static layer.
#pragma once
#include "wino_flex.hpp"
#include "wino_real_brackets.hpp"

namespace wino {

// T (ROWS x COLS, run-time, row-major) applied to a square S: ts = T S, tst = T S^T.
template <int ROWS, int COLS>
__device__ __forceinline__ void flex_left(const float* __restrict__ Tm, const float (&S)[COLS][COLS],
                                          float (&ts)[ROWS][COLS], float (&tst)[ROWS][COLS]) {
  static_for<0, ROWS>([&](auto i) {
    static_for<0, COLS>([&](auto b) {
      float a0 = 0.f, a1 = 0.f;
      static_for<0, COLS>([&](auto a) {
        const float c = Tm[decltype(i)::value * COLS + decltype(a)::value];
        a0 = __builtin_fmaf(c, S[a][b], a0);
        a1 = __builtin_fmaf(c, S[b][a], a1);
      });
      ts[i][b] = a0;
      tst[i][b] = a1;
    });
  });
}

// dT[i][b] = sum_j dR[i][j] tst[j][b] + dR[j][i] ts[j][b]   (this lane's share).
template <int ROWS, int COLS>
__device__ __forceinline__ void flex_matrix_grad(const float (&dR)[ROWS][ROWS],
                                                 const float (&ts)[ROWS][COLS],
                                                 const float (&tst)[ROWS][COLS],
                                                 float (&dT)[ROWS * COLS]) {
  static_for<0, ROWS>([&](auto i) {
    static_for<0, COLS>([&](auto b) {
      float acc = 0.f;
      static_for<0, ROWS>([&](auto j) {
        acc = __builtin_fmaf(dR[i][j], tst[j][b], acc);
        acc = __builtin_fmaf(dR[j][i], ts[j][b], acc);
      });
      dT[decltype(i)::value * COLS + decltype(b)::value] = acc;
    });
  });
}

// dS = T^T dR T.
template <int ROWS, int COLS>
__device__ __forceinline__ void flex_input_grad(const float* __restrict__ Tm,
                                                const float (&dR)[ROWS][ROWS],
                                                float (&dS)[COLS][COLS]) {
  float tmp[COLS][ROWS];
  static_for<0, COLS>([&](auto a) {
    static_for<0, ROWS>([&](auto j) {
      float acc = 0.f;
      static_for<0, ROWS>([&](auto i) {
        acc = __builtin_fmaf(Tm[decltype(i)::value * COLS + decltype(a)::value], dR[i][j], acc);
      });
      tmp[a][j] = acc;
    });
  });
  static_for<0, COLS>([&](auto a) {
    static_for<0, COLS>([&](auto b) {
      float acc = 0.f;
      static_for<0, ROWS>([&](auto j) {
        acc = __builtin_fmaf(tmp[a][j], Tm[decltype(j)::value * COLS + decltype(b)::value], acc);
      });
      dS[a][b] = acc;
    });
  });
}

// Sum of v[i] over the 256 lanes of the work group, in a fixed order (xor tree
// inside a wave, then wave 0 + 1 + 2 + 3), written to row[i] by lane i.
template <int CNT>
__device__ __forceinline__ void block_sum_to_row(const float (&v)[CNT], float* __restrict__ row) {
  __shared__ float s_red[4][CNT];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  static_for<0, CNT>([&](auto i) {
    float x = v[decltype(i)::value];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    if (lane == 0) s_red[wave][decltype(i)::value] = x;
  });
  __syncthreads();
  if (threadIdx.x < CNT) {
    const int i = threadIdx.x;
    row[i] = ((s_red[0][i] + s_red[1][i]) + s_red[2][i]) + s_red[3][i];
  }
}

constexpr int kPartialStride = 64;   // floats per work group in the partial-sum arrays

// dY, M -> dM and the partial sums of dAPT (m x n).  s_in: what one code of the
// A_P bracket's input stands for (s_m1, or the scale of M in the canonical base).
template <int M, bool LEG, typename MT>
__global__ __launch_bounds__(256) void k_fbwd_output(const MT* __restrict__ Mq,
                                                     const float* __restrict__ dy,
                                                     float* __restrict__ dM,
                                                     float* __restrict__ part, Geometry g,
                                                     FlexMats fm, StageMults mu, float s_in) {
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
  float S[n][n];
  static_for<0, n>([&](auto i) { static_for<0, n>([&](auto j) { S[i][j] = (float)xi[i][j] * s_in; }); });
  float dR[M][M];
  static_for<0, M>([&](auto i) {
    static_for<0, M>([&](auto j) {
      const int h = ty * M + decltype(i)::value, w = tx * M + decltype(j)::value;
      dR[i][j] = (active && h < g.H && w < g.W) ? dy[(((long)b * g.H + h) * g.W + w) * g.K + k] : 0.f;
    });
  });
  float ts[M][n], tst[M][n], dT[M * n];
  flex_left<M, n>(fm.APT, S, ts, tst);
  flex_matrix_grad<M, n>(dR, ts, tst, dT);
  float dS[n][n];
  flex_input_grad<M, n>(fm.APT, dR, dS);
  if (active) {
    if constexpr (LEG) {
      float out[n][n];
      adjoint_bracket_f<TabF<M>::PinvT>(dS, out);
      static_for<0, n>([&](auto i) {
        static_for<0, n>([&](auto j) {
          dM[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] = out[i][j];
        });
      });
    } else {
      static_for<0, n>([&](auto i) {
        static_for<0, n>([&](auto j) {
          dM[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] = dS[i][j];
        });
      });
    }
  }
  block_sum_to_row<M * n>(dT, part + (long)blockIdx.x * kPartialStride);
}

// dU, x -> per-tile dX [a*n+b][t][c] and the partial sums of dBPT (n x n).
// s_in: what one code of the B_P bracket's input stands for (s_x1, or s_x).
template <int M, bool LEG>
__device__ __forceinline__ void fbwd_input_body(const int8_t* __restrict__ x,
                                                const float* __restrict__ dU,
                                                float* __restrict__ dXt, float* __restrict__ part,
                                                const Geometry& g, const FlexMats& fm,
                                                const StageMults& mu, float s_in, unsigned block) {
  constexpr int n = M + 2;
  using TB = Tab<M>;
  const long total = (long)g.T * g.C;
  const long gid = (long)block * 256 + threadIdx.x;
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
  float S[n][n], dR[n][n];
  static_for<0, n>([&](auto i) {
    static_for<0, n>([&](auto j) {
      S[i][j] = (float)xi[i][j] * s_in;
      dR[i][j] = active ? dU[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] : 0.f;
    });
  });
  float dT[n * n];
  {
    float ts[n][n], tst[n][n];
    flex_left<n, n>(fm.BPT, S, ts, tst);
    flex_matrix_grad<n, n>(dR, ts, tst, dT);
  }
  float dS[n][n];
  flex_input_grad<n, n>(fm.BPT, dR, dS);
  if (active) {
    if constexpr (LEG) {
      float out[n][n];
      adjoint_bracket_f<TabF<M>::PinvT>(dS, out);
      static_for<0, n>([&](auto i) {
        static_for<0, n>([&](auto j) {
          dXt[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] = out[i][j];
        });
      });
    } else {
      static_for<0, n>([&](auto i) {
        static_for<0, n>([&](auto j) {
          dXt[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] = dS[i][j];
        });
      });
    }
  }
  block_sum_to_row<n * n>(dT, part + (long)block * kPartialStride);
}

// dV, w -> dw [k][c][3][3] and the partial sums of dGP (n x 3).
template <int M, bool LEG>
__device__ __forceinline__ void fbwd_weight_body(const int8_t* __restrict__ w,
                                                 float* __restrict__ dV,
                                                 float* __restrict__ dw, float* __restrict__ part,
                                                 const Geometry& g, const FlexMats& fm, float s_w,
                                                 unsigned block, int parts) {
  constexpr int n = M + 2;
  const long total = (long)g.K * g.C;
  const long gid = (long)block * 256 + threadIdx.x;
  const bool active = gid < total;
  float S[3][3];
  static_for<0, 3>([&](auto a) {
    static_for<0, 3>([&](auto bb) {
      S[a][bb] = active ? (float)w[gid * 9 + decltype(a)::value * 3 + decltype(bb)::value] * s_w : 0.f;
    });
  });
  float dR[n][n];
  {
    float v[n][n];
    load_summed_dv<n>(dV, total, gid, parts, active, v);
    if constexpr (LEG) {
      adjoint_bracket_f<TabF<M>::Pinv>(v, dR);      // V = P^{-1} W1 P^{-T}
    } else {
      static_for<0, n>([&](auto i) { static_for<0, n>([&](auto j) { dR[i][j] = v[i][j]; }); });
    }
  }
  float ts[n][3], tst[n][3], dT[n * 3];
  flex_left<n, 3>(fm.GP, S, ts, tst);
  flex_matrix_grad<n, 3>(dR, ts, tst, dT);
  float dS[3][3];
  flex_input_grad<n, 3>(fm.GP, dR, dS);
  if (active) {
    static_for<0, 3>([&](auto a) {
      static_for<0, 3>([&](auto bb) {
        dw[gid * 9 + decltype(a)::value * 3 + decltype(bb)::value] = dS[a][bb];
      });
    });
  }
  block_sum_to_row<n * 3>(dT, part + (long)block * kPartialStride);
}

// The input and the filter bracket are independent of each other: one launch, the first
// nb_w work groups take filters (few, and the longer chain of loads where dV comes in
// parts: they start first), the rest (tile, channel) items.
template <int M, bool LEG>
__global__ __launch_bounds__(256, (M <= 4 ? 4 : 1)) void k_fbwd_input_weight(
    const int8_t* __restrict__ x, const float* __restrict__ dU, float* __restrict__ dXt,
    float* __restrict__ part_in, const int8_t* __restrict__ w, float* __restrict__ dV,
    float* __restrict__ dw, float* __restrict__ part_w, Geometry g, FlexMats fm, StageMults mu,
    float s_in, float s_w, unsigned nb_w, int parts) {
  if (blockIdx.x < nb_w)
    fbwd_weight_body<M, LEG>(w, dV, dw, part_w, g, fm, s_w, blockIdx.x, parts);
  else
    fbwd_input_body<M, LEG>(x, dU, dXt, part_in, g, fm, mu, s_in, blockIdx.x - nb_w);
}

// dx[b][h][w][c] from per-tile gradients: tile ty reads input rows ty*M - 1 ... ty*M + M,
// so pixel row h is local row (h+1) % M of tile (h+1) / M and, when that is 0 or 1,
// also local row M + (h+1) % M of the tile above; columns alike.  The (at most four)
// contributions are added in a fixed order.
template <int M>
__global__ __launch_bounds__(256) void k_bwd_tile_sum(const float* __restrict__ dXt,
                                                      float* __restrict__ dx, Geometry g) {
  using v4f = __attribute__((ext_vector_type(4))) float;
  constexpr int n = M + 2;
  // one lane per four channels of a pixel (C is a multiple of 16); blockIdx.y = image row
  const int c4s = g.C / 4;
  const unsigned e = blockIdx.x * 256 + threadIdx.x;       // index in the row: w * c4s + c4
  if (e >= (unsigned)(g.W * c4s)) return;
  const int w = (int)(e / (unsigned)c4s), c = 4 * (int)(e - (unsigned)w * c4s);
  const long row = (long)blockIdx.y + (long)blockIdx.z * 65535;   // b * H + h
  if (row >= (long)g.N * g.H) return;
  const int b = (int)(row / g.H), h = (int)(row - (long)b * g.H);
  const long TC = (long)g.T * g.C;
  const int ty1 = (h + 1) / M, i1 = (h + 1) % M;
  const int tx1 = (w + 1) / M, j1 = (w + 1) % M;
  v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int dyv = 0; dyv < 2; ++dyv) {
    const int ty = ty1 - dyv, i = i1 + dyv * M;
    if (ty < 0 || ty >= g.TH || i >= n) continue;
#pragma unroll
    for (int dxv = 0; dxv < 2; ++dxv) {
      const int tx = tx1 - dxv, j = j1 + dxv * M;
      if (tx < 0 || tx >= g.TW || j >= n) continue;
      const long t = ((long)b * g.TH + ty) * g.TW + tx;
      acc += *reinterpret_cast<const v4f*>(dXt + (long)(i * n + j) * TC + t * g.C + c);
    }
  }
  *reinterpret_cast<v4f*>(dx + (row * g.W + w) * g.C + c) = acc;
}

template <int M>
hipError_t PerMFlexBwd<M>::output(const Geometry& g, bool leg, const void* Mq, int m_bits,
                                  const float* dy, float* dM, float* part, const FlexMats& fm,
                                  const StageMults& mu, float s_in, hipStream_t st) {
  const dim3 grid((unsigned)(((long)g.T * g.K + 255) / 256)), bs(256);
#define WINO_FBWD_OUT(LEGV, MTV)                                                                 \
  wino_launch((k_fbwd_output<M, LEGV, MTV>), grid, bs, st, static_cast<const MTV*>(Mq), dy, dM, \
              part, g, fm, mu, s_in)
  if (leg) {
    if (m_bits == 8) WINO_FBWD_OUT(true, int8_t);
    else if (m_bits == 9) WINO_FBWD_OUT(true, int16_t);
    else WINO_FBWD_OUT(true, int32_t);
  } else {
    if (m_bits == 8) WINO_FBWD_OUT(false, int8_t);
    else if (m_bits == 9) WINO_FBWD_OUT(false, int16_t);
    else WINO_FBWD_OUT(false, int32_t);
  }
#undef WINO_FBWD_OUT
  return hipGetLastError();
}

template <int M>
hipError_t PerMFlexBwd<M>::input_weight(const Geometry& g, bool leg, const int8_t* x,
                                        const float* dU, float* dXt, float* part_in,
                                        const int8_t* w, float* dV, float* dw,
                                        float* part_w, const FlexMats& fm, const StageMults& mu,
                                        float s_in, float s_w, hipStream_t st) {
  const unsigned nb_in = (unsigned)(((long)g.T * g.C + 255) / 256);
  const unsigned nb_w = (unsigned)(((long)g.K * g.C + 255) / 256);
  const dim3 grid(nb_in + nb_w), bs(256);
  const int parts = backward_dv_reader_parts(g);
  if (leg)
    wino_launch((k_fbwd_input_weight<M, true>), grid, bs, st, x, dU, dXt, part_in, w, dV, dw, part_w,
                g, fm, mu, s_in, s_w, nb_w, parts);
  else
    wino_launch((k_fbwd_input_weight<M, false>), grid, bs, st, x, dU, dXt, part_in, w, dV, dw,
                part_w, g, fm, mu, s_in, s_w, nb_w, parts);
  return hipGetLastError();
}

template <int M>
hipError_t PerMFlexBwd<M>::tile_sum(const Geometry& g, const float* dXt, float* dx,
                                    hipStream_t st) {
  const long rows = (long)g.N * g.H, per_row = (long)g.W * (g.C / 4);
  if (rows == 0 || per_row == 0) return hipSuccess;
  // grid: x over a row's (pixel, 4 channels) items, y and z over the image rows
  const long zs = (rows + 65534) / 65535;
  if (zs > 65535 || per_row >= (1L << 31)) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((per_row + 255) / 256), (unsigned)(rows < 65535 ? rows : 65535), (unsigned)zs);
  wino_launch((k_bwd_tile_sum<M>), grid, dim3(256), st, dXt, dx, g);
  return hipGetLastError();
}

}  // namespace wino
