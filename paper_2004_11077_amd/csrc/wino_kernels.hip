// Contraction kernel (gfx950 int8 MFMA) and the per-stage dispatchers.
#include "wino_kernels.hpp"

namespace wino {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// One symmetric cast: round to nearest even, clamp to +-qmax.
__device__ __forceinline__ int cast_code(float v, float qmax) {
  v = rintf(v);
  v = fminf(fmaxf(v, -qmax), qmax);
  return (int)v;
}

// ---------------------------------------------------------------------------
// Contraction: per Winograd point p, M[p][t][k] = sum_c U[p][t][c] V[p][k][c].
// One wave computes a 32(k) x 32(t) block with the 32x32x32 int8 MFMA; the A
// operand is V (rows k), the B operand U (rows t), so that a lane ends up with
// four consecutive k of one tile per accumulator quad.
// ---------------------------------------------------------------------------
template <typename MT>
__global__ __launch_bounds__(256) void k_contract(const int8_t* __restrict__ U,
                                                  const int8_t* __restrict__ V,
                                                  MT* __restrict__ Mo, int T, int C, int K,
                                                  int tblocks, float mult, float qmax) {
  const int p = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int tb = blockIdx.x % tblocks, kb = blockIdx.x / tblocks;
  const int t0 = tb * 64 + (wave & 1) * 32;
  const int k0 = kb * 64 + (wave >> 1) * 32;
  if (t0 >= T || k0 >= K) return;          // whole wave out of range
  const int r = lane & 31, h = lane >> 5;
  const int t = t0 + r, k = k0 + r;
  const int tl = t < T ? t : T - 1;        // clamp loads, mask stores
  const int kl = k < K ? k : K - 1;
  const int8_t* up = U + ((long)p * T + tl) * C + h * 16;
  const int8_t* vp = V + ((long)p * K + kl) * C + h * 16;
  v16i acc = {};
  for (int c0 = 0; c0 < C; c0 += 32) {
    v4i a = {}, bq = {};
    if (c0 + h * 16 < C) {
      a = *reinterpret_cast<const v4i*>(vp + c0);
      bq = *reinterpret_cast<const v4i*>(up + c0);
    }
    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, bq, acc, 0, 0, 0);
  }
  // acc[4*g+v] = D[row = 8*g + 4*h + v][col = r]  ->  k = k0 + row, tile t0 + r
  if (t >= T) return;
  MT* mrow = Mo + ((long)p * T + t) * K;
#pragma unroll
  for (int gq = 0; gq < 4; ++gq) {
    const int kk = k0 + 8 * gq + 4 * h;
    if (kk >= K) continue;
    int q[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      if constexpr (sizeof(MT) == 4)
        q[v] = acc[4 * gq + v];
      else
        q[v] = cast_code((float)acc[4 * gq + v] * mult, qmax);
    }
    if constexpr (sizeof(MT) == 1) {
      uint32_t pk = ((uint32_t)q[0] & 0xffu) | (((uint32_t)q[1] & 0xffu) << 8) |
                    (((uint32_t)q[2] & 0xffu) << 16) | (((uint32_t)q[3] & 0xffu) << 24);
      *reinterpret_cast<uint32_t*>(mrow + kk) = pk;
    } else if constexpr (sizeof(MT) == 2) {
      uint2 pk;
      pk.x = ((uint32_t)q[0] & 0xffffu) | ((uint32_t)q[1] << 16);
      pk.y = ((uint32_t)q[2] & 0xffffu) | ((uint32_t)q[3] << 16);
      *reinterpret_cast<uint2*>(mrow + kk) = pk;
    } else {
      int4 pk = make_int4(q[0], q[1], q[2], q[3]);
      *reinterpret_cast<int4*>(mrow + kk) = pk;
    }
  }
}

hipError_t launch_weight_transform(const Geometry& g, bool leg, const int8_t* w, int8_t* V,
                                   const StageMults& mu, hipStream_t st) {
  if ((long)g.K * g.C == 0) return hipSuccess;
  switch (g.m) {
    case 2: return PerM<2>::weight(g, leg, w, V, mu, st);
    case 4: return PerM<4>::weight(g, leg, w, V, mu, st);
    case 6: return PerM<6>::weight(g, leg, w, V, mu, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_input_transform(const Geometry& g, bool leg, const int8_t* x, int8_t* U,
                                  const StageMults& mu, hipStream_t st) {
  if ((long)g.T * g.C == 0) return hipSuccess;
  switch (g.m) {
    case 2: return PerM<2>::input(g, leg, x, U, mu, st);
    case 4: return PerM<4>::input(g, leg, x, U, mu, st);
    case 6: return PerM<6>::input(g, leg, x, U, mu, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_contract(const Geometry& g, const int8_t* U, const int8_t* V, void* Mo,
                           int m_bits, float mult, hipStream_t st) {
  if ((long)g.T * g.K == 0) return hipSuccess;
  const int n = g.m + 2;
  const int tblocks = (g.T + 63) / 64, kblocks = (g.K + 63) / 64;
  dim3 grid((unsigned)(tblocks * kblocks), (unsigned)(n * n));
  if (m_bits == 8)
    hipLaunchKernelGGL((k_contract<int8_t>), grid, dim3(256), 0, st, U, V, (int8_t*)Mo, g.T, g.C,
                       g.K, tblocks, mult, 127.f);
  else if (m_bits == 9)
    hipLaunchKernelGGL((k_contract<int16_t>), grid, dim3(256), 0, st, U, V, (int16_t*)Mo, g.T,
                       g.C, g.K, tblocks, mult, 255.f);
  else
    hipLaunchKernelGGL((k_contract<int32_t>), grid, dim3(256), 0, st, U, V, (int32_t*)Mo, g.T,
                       g.C, g.K, tblocks, mult, 0.f);
  return hipGetLastError();
}

hipError_t launch_output_transform(const Geometry& g, bool leg, const void* Mq, int m_bits,
                                   void* y, int out_type, bool relu, const StageMults& mu,
                                   hipStream_t st) {
  if ((long)g.T * g.K == 0) return hipSuccess;
  switch (g.m) {
    case 2: return PerM<2>::output(g, leg, Mq, m_bits, y, out_type, relu, mu, st);
    case 4: return PerM<4>::output(g, leg, Mq, m_bits, y, out_type, relu, mu, st);
    case 6: return PerM<6>::output(g, leg, Mq, m_bits, y, out_type, relu, mu, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace wino
