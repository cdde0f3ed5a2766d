// Contraction and output transform in ONE kernel (gfx950): the contraction
// result M (Hadamard product summed over the input channels, cast to
// bits_hadamard) never leaves the compute unit; only U, V and y touch HBM.
//
//   M[p][t][k] = cast( sum_c U[p][t][c] V[p][k][c] )       int8 MFMA, int32 accumulation
//   y          = output bracket of eq. 3 / eq. 4 applied to M[.][t][k]
//
// A work group of 4 waves owns TB tiles x KB output channels and ALL n*n
// Winograd points of that block, because the output bracket of a (tile, k) item
// needs every point.
//
// Phase 1 (contraction).  Wave w takes the points w, w + 4, ...; for each it
// runs the complete channel sum of the TB x KB block on the 16x16x64 int8 MFMA,
// with both operands loaded straight from global memory into the instruction's
// register layout (lane (j, s) of a 16-row fragment holds bytes 16 s .. 16 s + 15
// of a 64-channel chunk of row j).  Waves work on different points, so every
// operand byte enters the compute unit once per work group and no staging
// through LDS and no barrier is needed; the loads run DEPTH - 1 chunks ahead of
// the MFMAs.  A finished point is cast in registers and parked in LDS as
// M_s[p][tile][k].
// Phase 2 (output transform).  After one barrier every lane takes (tile, k)
// items, reads the n*n codes of its item from LDS and runs the same integer
// brackets and casts as the stand-alone output-transform kernel.
//
// Two work groups share a compute unit (LDS <= 80 KB each), so the matrix-pipe
// phase of one overlaps the vector-ALU phase of the other.  The block shape sets
// the operand bytes loaded per multiply-accumulate, TB KB / (TB + KB); it is
// bounded by the LDS that M_s needs, n*n TB KB sizeof(code).
//
// Work-group ids go round-robin over the 8 XCDs (each with its own L2): XCD x
// takes the tile blocks tb = x (mod 8) with all their k blocks, so the U rows
// of a tile block are fetched into one L2 only.
#pragma once
#include "wino_transforms.hpp"

namespace wino {

// One cast kept in its biased float form 1.5 * 2^23 + q: the code sits, in two's complement,
// in the low bits of the returned pattern, so packing needs only its low byte (or half).
__device__ __forceinline__ uint32_t co_cast_biased(float v, float mult, float qmax) {
  float t = __builtin_fmaf(v, mult, kMagic);
  t = __builtin_amdgcn_fmed3f(t, kMagic - qmax, kMagic + qmax);
  return __float_as_uint(t);
}

constexpr int kCoWaves = 4;
constexpr int kCoChunk = 64;      // channels per MFMA (16x16x64)
constexpr int kCoDepth = 3;       // operand chunks in flight per wave (one being consumed)

// Block shapes.  S: small problems (many work groups).  L: the largest block
// whose M_s still lets two work groups share a compute unit.
template <int M, typename MT, bool LARGE>
struct CoShape {
  static constexpr int n2 = (M + 2) * (M + 2);
  static constexpr int TB = !LARGE ? 16 : (n2 * 32 * 32 * (int)sizeof(MT) <= 80 * 1024 ? 32 : 16);
  static constexpr int KB = !LARGE ? 32 : (n2 * TB * 64 * (int)sizeof(MT) <= 80 * 1024 ? 64 : 32);
};

template <int M, bool LEG, typename MT, int OUT, bool PP, int TB, int KB>
__global__ __launch_bounds__(256, 2) void k_contract_out(const int8_t* __restrict__ U,
                                                         const int8_t* __restrict__ V,
                                                         void* __restrict__ yv, Geometry g,
                                                         StageMults mu, MultTable mm, ShiftTable sh,
                                                         int relu, int tblocks, int kblocks) {
  constexpr int n = M + 2, n2 = n * n;
  constexpr int NTB = TB / 16, NKB = KB / 16;       // 16-row fragments per operand
  constexpr int NPW = (n2 + kCoWaves - 1) / kCoWaves;
  static_assert(n2 % kCoWaves == 0);
  constexpr float QM = sizeof(MT) == 1 ? 127.f : 255.f;
  using TBL = Tab<M>;
  __shared__ __attribute__((aligned(16))) MT M_s[n2 * TB * KB];
  __shared__ int4 s_tile[TB];                        // {image, first output row, first column, exists}

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int kbi = slot % kblocks, tbi = (slot / kblocks) * 8 + xcd;
  if (tbi >= tblocks) return;                        // block-uniform
  const int t0 = tbi * TB, k0 = kbi * KB;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: indexes kernel-argument tables
  const int jl = lane & 15, seg = lane >> 4;
  if (tid < TB) {
    const int t = t0 + tid;
    const int tx = t % g.TW;
    const int ty = (t / g.TW) % g.TH;
    const int b = t / (g.TW * g.TH);
    s_tile[tid] = make_int4(b, ty * M, tx * M, t < g.T ? 1 : 0);
  }

  // ---- phase 1: contraction of the wave's points --------------------------------------
  // Rows past the last tile / output channel are read from the last existing row; their
  // results land in items that phase 2 skips.  Lane offsets fit 32 bits (64 rows of C <= 2^20).
  const int C = g.C;
  uint32_t offA[NKB], offB[NTB];
#pragma unroll
  for (int i = 0; i < NKB; ++i)
    offA[i] = (uint32_t)(min(k0 + i * 16 + jl, g.K - 1) - k0) * (uint32_t)C + seg * 16;
#pragma unroll
  for (int i = 0; i < NTB; ++i)
    offB[i] = (uint32_t)(min(t0 + i * 16 + jl, g.T - 1) - t0) * (uint32_t)C + seg * 16;
  const int nchunks = (C + kCoChunk - 1) / kCoChunk;
  const int nunits = NPW * nchunks;                  // (point, chunk) pairs of this wave, point-major

  struct Frag {
    v4i a[NKB], b[NTB];
  };
  Frag ring[kCoDepth];
  int lpi = 0, lci = 0;                              // next unit to load
  auto load = [&](Frag& f) {
    const int p = lpi * kCoWaves + wave;
    const int c0 = lci * kCoChunk;
    const int8_t* Vp = V + ((long)p * g.K + k0) * C + c0;   // wave-uniform bases
    const int8_t* Up = U + ((long)p * g.T + t0) * C + c0;
    const bool ok = c0 + seg * 16 < C;               // false only inside a partial last chunk
#pragma unroll
    for (int i = 0; i < NKB; ++i)
      f.a[i] = ok ? *reinterpret_cast<const v4i*>(Vp + offA[i]) : v4i{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < NTB; ++i)
      f.b[i] = ok ? *reinterpret_cast<const v4i*>(Up + offB[i]) : v4i{0, 0, 0, 0};
    if (++lci == nchunks) lci = 0, ++lpi;
  };

  v4i acc[NKB][NTB];
  int cpi = 0, cci = 0;                              // unit being consumed
  auto consume = [&](const Frag& f) {
    if (cci == 0) {
#pragma unroll
      for (int i = 0; i < NKB; ++i)
#pragma unroll
        for (int j = 0; j < NTB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f.a[i], f.b[j], v4i{0, 0, 0, 0}, 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < NKB; ++i)
#pragma unroll
        for (int j = 0; j < NTB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
    }
    if (++cci == nchunks) {
      // acc[i][j][v] = D[k = 16 i + 4 seg + v][tile = 16 j + jl]: cast, pack the four
      // consecutive k of a tile, park as M_s[p][tile][k]
      const int p = cpi * kCoWaves + wave;
      const float mult = PP ? mm.v[p] : mm.v[0];
#pragma unroll
      for (int i = 0; i < NKB; ++i)
#pragma unroll
        for (int j = 0; j < NTB; ++j) {
          uint32_t q[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) q[v] = co_cast_biased((float)acc[i][j][v], mult, QM);
          MT* dst = M_s + (p * TB + j * 16 + jl) * KB + i * 16 + 4 * seg;
          if constexpr (sizeof(MT) == 1) {
            const uint32_t lo = __builtin_amdgcn_perm(q[1], q[0], 0x0c0c0400u);
            const uint32_t hi = __builtin_amdgcn_perm(q[3], q[2], 0x04000c0cu);
            *reinterpret_cast<uint32_t*>(dst) = lo | hi;
          } else {
            uint2 pk;
            pk.x = __builtin_amdgcn_perm(q[1], q[0], 0x05040100u);
            pk.y = __builtin_amdgcn_perm(q[3], q[2], 0x05040100u);
            *reinterpret_cast<uint2*>(dst) = pk;
          }
        }
      cci = 0, ++cpi;
    }
  };

  static_for<0, kCoDepth - 1>([&](auto d) {
    if (decltype(d)::value < nunits) load(ring[decltype(d)::value]);
  });
  for (int u0 = 0; u0 < nunits; u0 += kCoDepth) {
    static_for<0, kCoDepth>([&](auto d) {
      constexpr int D = decltype(d)::value;
      const int u = u0 + D;
      if (u + kCoDepth - 1 < nunits) load(ring[(D + kCoDepth - 1) % kCoDepth]);
      if (u < nunits) consume(ring[D]);
    });
  }
  __syncthreads();

  // ---- phase 2: output transform of TB x KB items ---------------------------------------
  constexpr int64_t IN_MAX = (sizeof(MT) == 1 ? 127 : 255) << (PP ? kMaxMShift : 0);
#pragma unroll 1
  for (int it = 0; it < TB * KB / 256; ++it) {
    const int item = it * 256 + tid;
    const int tl = item / KB, kl = item - tl * KB;
    const int k = k0 + kl;
    const int4 ti = s_tile[tl];
    if (!ti.w || k >= g.K) continue;
    const int ty_m = ti.y, tx_m = ti.z;
    int mi[n][n];
    static_for<0, n>([&](auto i) {
      static_for<0, n>([&](auto j) {
        constexpr int P = decltype(i)::value * n + decltype(j)::value;
        mi[i][j] = (int)M_s[(P * TB + tl) * KB + kl];
        if constexpr (PP) mi[i][j] <<= sh.v[P];
      });
    });
    const long ybase = (((long)ti.x * g.H + ty_m) * g.W + tx_m) * g.K + k;
    const int wk = g.W * g.K;
    auto finish = [&]<const IMat& FT, int64_t FIN>(auto& num) {
      static_for<0, M>([&](auto i) {
        static_for<0, M>([&](auto j) {
          constexpr int I = decltype(i)::value, J = decltype(j)::value;
          if (ty_m + I < g.H && tx_m + J < g.W) {
            const int rel = I * wk + J * g.K;
            if constexpr (OUT == 0) {
              float v = to_float_approx(entry<FT, FIN, I, J>(num[i][j])) * mu.outer.v[I * M + J];
              __builtin_nontemporal_store(relu ? fmaxf(v, 0.f) : v, static_cast<float*>(yv) + ybase + rel);
            } else {
              int v = cast_code((float)entry<FT, FIN, I, J>(num[i][j]), mu.outer.v[I * M + J], 127.f);
              __builtin_nontemporal_store((int8_t)(relu ? max(v, 0) : v),
                                          static_cast<int8_t*>(yv) + ybase + rel);
            }
          }
        });
      });
    };
    if constexpr (LEG) {
      acc_t<TBL::PinvT, IN_MAX> num1[n][n];
      sandwich<TBL::PinvT, IN_MAX>(mi, num1);
      int m1[n][n];
      cast_result<TBL::PinvT, IN_MAX>(num1, mu.inner, 127.f, m1);
      acc_t<TBL::APT, 127> num2[M][M];
      sandwich<TBL::APT, 127>(m1, num2);
      finish.template operator()<TBL::APT, 127>(num2);
    } else {
      acc_t<TBL::AT, IN_MAX> num[M][M];
      sandwich<TBL::AT, IN_MAX>(mi, num);
      finish.template operator()<TBL::AT, IN_MAX>(num);
    }
  }
}

// shape: 0 = chosen from the problem size, 1 = small blocks, 2 = large blocks
template <int M, bool LEG, typename MT, int OUT, bool PP, bool LARGE>
static hipError_t conout_launch(const Geometry& g, const int8_t* U, const int8_t* V, void* y,
                                bool relu, const StageMults& mu, const MultTable& mm,
                                const ShiftTable& sh, hipStream_t st) {
  constexpr int TB = CoShape<M, MT, LARGE>::TB, KB = CoShape<M, MT, LARGE>::KB;
  const int tblocks = (g.T + TB - 1) / TB, kblocks = (g.K + KB - 1) / KB;
  const long nblocks = (long)((tblocks + 7) / 8) * 8 * kblocks;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  wino_launch((k_contract_out<M, LEG, MT, OUT, PP, TB, KB>), dim3((unsigned)nblocks), dim3(256), st,
              U, V, y, g, mu, mm, sh, relu ? 1 : 0, tblocks, kblocks);
  return hipGetLastError();
}

template <int M, bool LEG, typename MT, int OUT, bool PP>
static hipError_t conout_shape(const Geometry& g, const int8_t* U, const int8_t* V, void* y,
                               bool relu, const StageMults& mu, const MultTable& mm,
                               const ShiftTable& sh, int shape, hipStream_t st) {
  using L = CoShape<M, MT, true>;
  bool large = shape == 2;
  if (shape == 0) {
    // large blocks once they still give every compute unit its two work groups
    const long nl = (long)((g.T + L::TB - 1) / L::TB) * ((g.K + L::KB - 1) / L::KB);
    large = nl >= 2 * 256;
  }
  return large ? conout_launch<M, LEG, MT, OUT, PP, true>(g, U, V, y, relu, mu, mm, sh, st)
               : conout_launch<M, LEG, MT, OUT, PP, false>(g, U, V, y, relu, mu, mm, sh, st);
}

template <int M, bool LEG, typename MT>
static hipError_t conout_mt(const Geometry& g, const int8_t* U, const int8_t* V, void* y,
                            int out_type, bool relu, const StageMults& mu, const MultTable& mm,
                            const ShiftTable* sh, int shape, hipStream_t st) {
  const ShiftTable none{};
  if (out_type != 0 && out_type != 2) return hipErrorInvalidValue;
  if (sh)
    return out_type == 0 ? conout_shape<M, LEG, MT, 0, true>(g, U, V, y, relu, mu, mm, *sh, shape, st)
                         : conout_shape<M, LEG, MT, 2, true>(g, U, V, y, relu, mu, mm, *sh, shape, st);
  return out_type == 0 ? conout_shape<M, LEG, MT, 0, false>(g, U, V, y, relu, mu, mm, none, shape, st)
                       : conout_shape<M, LEG, MT, 2, false>(g, U, V, y, relu, mu, mm, none, shape, st);
}

template <int M>
hipError_t PerMCO<M>::run(const Geometry& g, bool leg, const int8_t* U, const int8_t* V, void* y,
                          int m_bits, int out_type, bool relu, const StageMults& mu,
                          const MultTable& mm, const ShiftTable* sh, int shape, hipStream_t st) {
  if (m_bits == 8)
    return leg ? conout_mt<M, true, int8_t>(g, U, V, y, out_type, relu, mu, mm, sh, shape, st)
               : conout_mt<M, false, int8_t>(g, U, V, y, out_type, relu, mu, mm, sh, shape, st);
  if (m_bits == 9)
    return leg ? conout_mt<M, true, int16_t>(g, U, V, y, out_type, relu, mu, mm, sh, shape, st)
               : conout_mt<M, false, int16_t>(g, U, V, y, out_type, relu, mu, mm, sh, shape, st);
  return hipErrorInvalidValue;
}

}  // namespace wino
