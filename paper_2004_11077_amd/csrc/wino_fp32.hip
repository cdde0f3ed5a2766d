// fp32 path (bits_in = 32): the same four stages of eq. 3 / eq. 4 without any
// cast, on float tensors with the layouts of the int8 path (x NHWC, w KCRS,
// U [n*n][T][C], V [n*n][K][C], M [n*n][T][K], y NHWC).  It exists as the
// unquantised reference of the library (checked against fp64 to 1e-4); it is
// not tuned: one lane per item in the transforms, one lane per output in the
// contraction.  Tensors and the contraction are fp32; a Legendre bracket pair
// is evaluated in double between its fp32 input and its fp32 result (see
// bracket_d).
#include "wino_kernels.hpp"
#include "wino_real_brackets.hpp"

namespace wino {

template <int M, bool LEG>
__global__ __launch_bounds__(256) void k_weight_f32(const float* __restrict__ w,
                                                    float* __restrict__ V, Geometry g) {
  constexpr int n = M + 2;
  using TB = TabF<M>;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const long KC = (long)g.K * g.C;
  if (gid >= KC) return;
  float wi[3][3];
  rfor<0, 3>([&](auto a) {
    rfor<0, 3>([&](auto b) { wi[a][b] = w[gid * 9 + decltype(a)::value * 3 + decltype(b)::value]; });
  });
  float v[n][n];
  if constexpr (LEG) {
    double w1[n][n];
    bracket_d<TB::GP>(wi, w1);       // G_P W G_P^T
    bracket_d<TB::Pinv>(w1, v);      // P^{-1} ( . ) P^{-T}
  } else {
    bracket_f<TB::G>(wi, v);
  }
  rfor<0, n>([&](auto i) {
    rfor<0, n>([&](auto j) {
      V[(long)(decltype(i)::value * n + decltype(j)::value) * KC + gid] = v[i][j];
    });
  });
}

template <int M, bool LEG>
__global__ __launch_bounds__(256) void k_input_f32(const float* __restrict__ x,
                                                   float* __restrict__ U, Geometry g) {
  constexpr int n = M + 2;
  using TB = TabF<M>;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const long total = (long)g.T * g.C;
  if (gid >= total) return;
  const int t = (int)(gid / g.C);
  const int c = (int)(gid - (long)t * g.C);
  const int tx = t % g.TW;
  const int ty = (t / g.TW) % g.TH;
  const int b = t / (g.TW * g.TH);
  float xi[n][n];
  rfor<0, n>([&](auto a) {
    rfor<0, n>([&](auto bb) {
      const int h = ty * M - 1 + decltype(a)::value;
      const int ww = tx * M - 1 + decltype(bb)::value;
      float v = 0.f;
      if (h >= 0 && h < g.H && ww >= 0 && ww < g.W)
        v = x[(((long)b * g.H + h) * g.W + ww) * g.C + c];
      xi[a][bb] = v;
    });
  });
  float u[n][n];
  if constexpr (LEG) {
    double x1[n][n];
    bracket_d<TB::PinvT>(xi, x1);    // P^{-T} X P^{-1}
    bracket_d<TB::BPT>(x1, u);       // B_P^T ( . ) B_P
  } else {
    bracket_f<TB::BT>(xi, u);
  }
  rfor<0, n>([&](auto i) {
    rfor<0, n>([&](auto j) {
      U[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] = u[i][j];
    });
  });
}

// M[p][t][k] = sum_c U[p][t][c] V[p][k][c]; one lane per output, 16 (t) x 16 (k)
// outputs per work group with both operand panels staged through LDS.
__global__ __launch_bounds__(256) void k_contract_f32(const float* __restrict__ U,
                                                      const float* __restrict__ V,
                                                      float* __restrict__ Mo, int T, int C,
                                                      int K, int tblocks) {
  __shared__ float su[16][17], sv[16][17];
  const int p = blockIdx.y;
  const int tb = blockIdx.x % tblocks, kb = blockIdx.x / tblocks;
  const int tl = threadIdx.x >> 4, kl = threadIdx.x & 15;
  const int t = tb * 16 + tl, k = kb * 16 + kl;
  float acc = 0.f;
  for (int c0 = 0; c0 < C; c0 += 16) {
    // lane (row = tl, col = kl) loads one element of each panel
    const int tr = tb * 16 + tl, kr = kb * 16 + tl, cc = c0 + kl;
    su[tl][kl] = (tr < T && cc < C) ? U[((long)p * T + tr) * C + cc] : 0.f;
    sv[tl][kl] = (kr < K && cc < C) ? V[((long)p * K + kr) * C + cc] : 0.f;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 16; ++c) acc = __builtin_fmaf(su[tl][c], sv[kl][c], acc);
    __syncthreads();
  }
  if (t < T && k < K) Mo[((long)p * T + t) * K + k] = acc;
}

template <int M, bool LEG>
__global__ __launch_bounds__(256) void k_output_f32(const float* __restrict__ Mq,
                                                    float* __restrict__ y, Geometry g, int relu) {
  constexpr int n = M + 2;
  using TB = TabF<M>;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const long total = (long)g.T * g.K;
  if (gid >= total) return;
  const int t = (int)(gid / g.K);
  const int k = (int)(gid - (long)t * g.K);
  const int tx = t % g.TW;
  const int ty = (t / g.TW) % g.TH;
  const int b = t / (g.TW * g.TH);
  float mi[n][n];
  rfor<0, n>([&](auto i) {
    rfor<0, n>([&](auto j) {
      mi[i][j] = Mq[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid];
    });
  });
  float out[M][M];
  if constexpr (LEG) {
    double m1[n][n];
    bracket_d<TB::PinvT>(mi, m1);    // P^{-T} M P^{-1}
    bracket_d<TB::APT>(m1, out);     // A_P^T ( . ) A_P
  } else {
    bracket_f<TB::AT>(mi, out);
  }
  rfor<0, M>([&](auto i) {
    rfor<0, M>([&](auto j) {
      const int h = ty * M + decltype(i)::value;
      const int ww = tx * M + decltype(j)::value;
      if (h < g.H && ww < g.W) {
        const float v = out[i][j];
        y[(((long)b * g.H + h) * g.W + ww) * g.K + k] = relu ? fmaxf(v, 0.f) : v;
      }
    });
  });
}

static inline unsigned nblk(long items) { return (unsigned)((items + 255) / 256); }

template <int M>
static hipError_t stage_f32(int stage, const Geometry& g, bool leg, const float* a, const float* b,
                            float* out, bool relu, hipStream_t st) {
  switch (stage) {
    case 0:
      if (leg)
        wino_launch((k_weight_f32<M, true>), dim3(nblk((long)g.K * g.C)), dim3(256), st, a, out, g);
      else
        wino_launch((k_weight_f32<M, false>), dim3(nblk((long)g.K * g.C)), dim3(256), st, a, out, g);
      break;
    case 1:
      if (leg)
        wino_launch((k_input_f32<M, true>), dim3(nblk((long)g.T * g.C)), dim3(256), st, a, out, g);
      else
        wino_launch((k_input_f32<M, false>), dim3(nblk((long)g.T * g.C)), dim3(256), st, a, out, g);
      break;
    case 2: {
      const int tblocks = (g.T + 15) / 16, kblocks = (g.K + 15) / 16;
      wino_launch(k_contract_f32, dim3((unsigned)(tblocks * kblocks), (unsigned)((M + 2) * (M + 2))),
                         dim3(256), st, a, b, out, g.T, g.C, g.K, tblocks);
      break;
    }
    default:
      if (leg)
        wino_launch((k_output_f32<M, true>), dim3(nblk((long)g.T * g.K)), dim3(256), st, a, out, g, relu ? 1 : 0);
      else
        wino_launch((k_output_f32<M, false>), dim3(nblk((long)g.T * g.K)), dim3(256), st, a, out, g, relu ? 1 : 0);
  }
  return hipGetLastError();
}

hipError_t launch_stage_f32(int stage, const Geometry& g, bool legendre, const float* a,
                            const float* b, float* out, bool relu, hipStream_t st) {
  const long items = stage == 0 ? (long)g.K * g.C : stage == 1 ? (long)g.T * g.C : (long)g.T * g.K;
  if (items == 0) return hipSuccess;
  switch (g.m) {
    case 2: return stage_f32<2>(stage, g, legendre, a, b, out, relu, st);
    case 4: return stage_f32<4>(stage, g, legendre, a, b, out, relu, st);
    case 6: return stage_f32<6>(stage, g, legendre, a, b, out, relu, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace wino
