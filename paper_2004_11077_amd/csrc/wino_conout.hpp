// Contraction and output transform in ONE kernel (gfx950): the contraction
// result M (Hadamard product summed over the input channels, cast to
// bits_hadamard) never leaves the compute unit; only U, V and y touch HBM.
//
//   M[p][t][k] = cast( sum_c U[p][t][c] V[p][k][c] )       int8 MFMA, int32 accumulation
//   y          = output bracket of eq. 3 / eq. 4 applied to M[.][t][k]
//
// A work group of NW waves owns TB tiles x KB output channels and ALL n*n
// Winograd points of that block, because the output bracket of a (tile, k) item
// needs every point.
//
// Phase 1 (contraction).  Wave w takes the points w, w + NW, ...; for each it
// runs the complete channel sum of the TB x KB block on the 16x16x64 int8 MFMA,
// with both operands loaded straight from global memory into the instruction's
// register layout (lane (j, s) of a 16-row fragment holds bytes 16 s .. 16 s + 15
// of a 64-channel chunk of row j).  With U and V stored in that order
// ("fragment order") a wave's load is one contiguous KiB; from row-major
// operands the four lanes of every quad touch four different rows, and the
// memory pipeline then runs at a quarter of its rate (measured: 10.5 TB/s of
// operand traffic chip-wide against 30 TB/s), so the transforms write fragment
// order for this kernel.  Waves work on different points, so every operand byte
// enters the compute unit once per work group and no staging through LDS and no
// barrier is needed; the loads run DEPTH - 1 units ahead of the MFMAs.  A
// finished point is cast in registers and parked in LDS as M_s[p][tile][k].
// Phase 2 (output transform).  After one barrier every lane takes (tile, k)
// items, reads the n*n codes of its item from LDS and runs the same integer
// brackets and casts as the stand-alone output-transform kernel.
//
// Two work groups share a compute unit (LDS <= 80 KB each).  The block shape sets
// the operand bytes loaded per multiply-accumulate, TB KB / (TB + KB); it is
// bounded by the LDS that M_s needs, n*n TB KB sizeof(code).
//
// Work-group ids go round-robin over the 8 XCDs (each with its own L2): XCD x
// takes the tile blocks tb = x (mod 8) with all their k blocks, so the U rows
// of a tile block are fetched into one L2 only.
#pragma once
#include "wino_transforms.hpp"

namespace wino {

constexpr int kCoChunk = 64;      // channels per MFMA step (16x16x64)

// Block shape: 32 tiles x 32 output channels where the codes of such a block fit 80 KB of LDS
// (two work groups per compute unit), else 16 x 32.  Measured on the 256-channel layer from
// 256 to 16384 tiles, this shape with eight waves and two operand units in flight was the
// fastest or within 5 % of the fastest of 16 x 32, 16 x 64, 32 x 32 and 32 x 64 blocks with 4,
// 8, 9, 12 or 16 waves and two or three units in flight.
template <int M, typename MT>
struct CoShape {
  static constexpr int n2 = (M + 2) * (M + 2);
  static constexpr int TB = n2 * 32 * 32 * (int)sizeof(MT) <= 80 * 1024 ? 32 : 16;
  static constexpr int KB = 32;
  static constexpr int NW = 8;       // waves per work group
  static constexpr int DEPTH = 2;    // operand units in flight per wave (one being consumed)
};

// NW waves per work group, WPE waves per SIMD that the register budget must allow, DEPTH
// operand units in flight per wave.
// FRAG: U and V are in MFMA-fragment order (wino_kernels.hpp), else rows [n*n][T or K][C].
template <int M, bool LEG, typename MT, int OUT, bool PP, bool FRAG, int TB, int KB, int NW, int WPE,
          int DEPTH>
__global__ __launch_bounds__(NW * 64, WPE) void k_contract_out(const int8_t* __restrict__ U,
                                                         const int8_t* __restrict__ V,
                                                         void* __restrict__ yv, Geometry g,
                                                         StageMults mu, MultTable mm, ShiftTable sh,
                                                         int relu, int tblocks, int kblocks) {
  constexpr int n = M + 2, n2 = n * n;
  constexpr int NTB = TB / 16, NKB = KB / 16;       // 16-row fragments per operand
  // All NW waves contract; the NT2 lanes of the first waves (a power of two) transform.
  constexpr int kCoWaves = NW, kCoDepth = DEPTH;
  constexpr int NT2 = (NW >= 16 ? 16 : NW >= 8 ? 8 : 4) * 64;
  static_assert(TB * KB % NT2 == 0);
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
    int tx, ty, b;
    tile_coords(g, min(t, g.T - 1), b, ty, tx);
    s_tile[tid] = make_int4(b, ty * M, tx * M, t < g.T ? 1 : 0);
  }

  // ---- phase 1: contraction of the wave's points --------------------------------------
  // The channel sum runs in units of 128 channels = two MFMA steps; the loads of a unit stay
  // in flight across the MFMAs of the units before it.  Every load of the loop is
  // unconditional and in bounds, so the loop body is straight-line code.  Rows past the last
  // tile / output channel are read from existing memory; their results land in items that
  // phase 2 skips.
  //
  // Fragment order (FRAG): a fragment of a 64-channel chunk is one contiguous KiB, lane l
  // reads bytes [16 l, 16 l + 16): a wave's load is one fully coalesced request with a scalar
  // base.  Chunks 2 u and 2 u + 1 form unit u; an odd chunk count leaves the last unit with
  // one MFMA step.  Channels past C are zeros in V, so no masking is needed.
  //
  // Rows (!FRAG): lane (j, s) of a 16-row fragment loads the 32 bytes [32 s, 32 s + 32) of
  // row j's 128-byte unit as two 16-byte pieces; piece h feeds MFMA step h (the MFMA's
  // reduction index may be any permutation of the channels as long as both operands use the
  // same one).  The four lanes of a quad read four different rows, which the memory pipeline
  // serves at a quarter of its rate: this form exists for operands in the documented row
  // layout and is not the fast path.  A partial last unit (C not a multiple of 128) reads the
  // 128-channel window that ENDS at C, and the pieces that belong to the unit before are
  // zeroed ahead of the MFMAs; a layer with C < 128 has one unit whose pieces are
  // [64 h + 16 s, + 16), clamped into the row and zeroed from C on (step 1 is skipped when
  // C <= 64).  Lane offsets fit 32 bits (64 rows of C <= 2^20).
  constexpr int kUnit = 2 * kCoChunk;
  const int C = g.C;
  const int nch = (C + kCoChunk - 1) / kCoChunk;     // 64-channel chunks
  const int nchunks = (C + kUnit - 1) / kUnit;       // units per point
  const int rem = C & (kUnit - 1);                   // rows: channels of a partial last unit
  const bool narrow = C < kUnit;
  const int lastc0 = rem ? max(C - kUnit, 0) : (nchunks - 1) * kUnit;
  int piece[2], keep[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int o = narrow ? h * kCoChunk + seg * 16 : seg * 32 + h * 16;
    piece[h] = min(o, C - 16);
    keep[h] = narrow ? (o < C ? -1 : 0) : (o >= kUnit - rem ? -1 : 0);
  }
  // is MFMA step 1 of the last unit of a point real?
  const bool last_has_two = FRAG ? (nch & 1) == 0 : C > kCoChunk;
  const int d1 = piece[1] - piece[0];
  uint32_t offA[NKB], offB[NTB];                     // rows: lane offsets inside the row block
  long fragA[NKB], fragB[NTB];                       // fragments: scalar offsets of the point's fragments
  const long rgV = (g.K + 15) >> 4, rgU = (g.T + 15) >> 4;
#pragma unroll
  for (int i = 0; i < NKB; ++i) {
    offA[i] = (uint32_t)(min(k0 + i * 16 + jl, g.K - 1) - k0) * (uint32_t)C + piece[0];
    fragA[i] = ((long)wave * rgV + min((long)(k0 >> 4) + i, rgV - 1)) * nch * 1024;
  }
#pragma unroll
  for (int i = 0; i < NTB; ++i) {
    offB[i] = (uint32_t)(min(t0 + i * 16 + jl, g.T - 1) - t0) * (uint32_t)C + piece[0];
    fragB[i] = ((long)wave * rgU + min((long)(t0 >> 4) + i, rgU - 1)) * nch * 1024;
  }
  const int NPW = (n2 - wave + NW - 1) / NW;         // points of this wave: wave, wave + NW, ...
  const int nunits = NPW * nchunks;                  // (point, unit) pairs of this wave, point-major

  struct Frag {
    v4i a[NKB][2], b[NTB][2];
  };
  Frag ring[kCoDepth];
  // next unit to load: row bases of its point (wave-uniform) and its channel window; past
  // the last unit the last one is loaded again (never consumed)
  const long vstep = FRAG ? (long)kCoWaves * rgV * nch * 1024 : (long)kCoWaves * g.K * C;
  const long ustep = FRAG ? (long)kCoWaves * rgU * nch * 1024 : (long)kCoWaves * g.T * C;
  const int8_t* vrow = FRAG ? V : V + ((long)wave * g.K + k0) * C;
  const int8_t* urow = FRAG ? U : U + ((long)wave * g.T + t0) * C;
  uint32_t lane16 = lane * 16;
  int lpi = 0, lci = 0;
  auto load = [&](Frag& f) {
    if constexpr (FRAG) {
      // made opaque here so that its zero-extension is formed in this block and the loads take
      // the form scalar base + 32-bit lane offset (no 64-bit vector adds)
      asm("" : "+v"(lane16));
      const long c0 = (long)(2 * lci) * 1024, c1 = (long)min(2 * lci + 1, nch - 1) * 1024;
#pragma unroll
      for (int i = 0; i < NKB; ++i) {
        f.a[i][0] = *reinterpret_cast<const v4i*>(vrow + fragA[i] + c0 + lane16);
        f.a[i][1] = *reinterpret_cast<const v4i*>(vrow + fragA[i] + c1 + lane16);
      }
#pragma unroll
      for (int i = 0; i < NTB; ++i) {
        f.b[i][0] = *reinterpret_cast<const v4i*>(urow + fragB[i] + c0 + lane16);
        f.b[i][1] = *reinterpret_cast<const v4i*>(urow + fragB[i] + c1 + lane16);
      }
    } else {
      const int c0 = lci == nchunks - 1 ? lastc0 : lci * kUnit;
      const int8_t* Vp = vrow + c0;
      const int8_t* Up = urow + c0;
#pragma unroll
      for (int i = 0; i < NKB; ++i) {
        f.a[i][0] = *reinterpret_cast<const v4i*>(Vp + offA[i]);
        f.a[i][1] = *reinterpret_cast<const v4i*>(Vp + offA[i] + d1);
      }
#pragma unroll
      for (int i = 0; i < NTB; ++i) {
        f.b[i][0] = *reinterpret_cast<const v4i*>(Up + offB[i]);
        f.b[i][1] = *reinterpret_cast<const v4i*>(Up + offB[i] + d1);
      }
    }
    if (lci + 1 < nchunks) {
      ++lci;
    } else if (lpi + 1 < NPW) {
      lci = 0, ++lpi, vrow += vstep, urow += ustep;
    }
  };

  v4i acc[NKB][NTB];
  int cpi = 0, cci = 0;                              // unit being consumed
  auto consume = [&](Frag& f) {
    const bool last = cci == nchunks - 1;
    if (!FRAG && last && rem) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < NKB; ++i) f.a[i][h] &= keep[h];
#pragma unroll
        for (int i = 0; i < NTB; ++i) f.b[i][h] &= keep[h];
      }
    }
    // the first unit of a point starts from the constant zero (wave-uniform branch): no
    // accumulator is cleared between points
    if (cci == 0) {
#pragma unroll
      for (int i = 0; i < NKB; ++i)
#pragma unroll
        for (int j = 0; j < NTB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f.a[i][0], f.b[j][0], v4i{0, 0, 0, 0}, 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < NKB; ++i)
#pragma unroll
        for (int j = 0; j < NTB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f.a[i][0], f.b[j][0], acc[i][j], 0, 0, 0);
    }
    if (!last || last_has_two) {
#pragma unroll
      for (int i = 0; i < NKB; ++i)
#pragma unroll
        for (int j = 0; j < NTB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f.a[i][1], f.b[j][1], acc[i][j], 0, 0, 0);
    }
    ++cci;
    if (last) {
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
          for (int v = 0; v < 4; ++v) q[v] = cast_biased((float)acc[i][j][v], mult, QM);
          // the four-code group index inside a tile's row is XOR-ed with the tile's low
          // bits: the 16 tiles a store covers then fall on distinct LDS banks
          MT* dst = M_s + (p * TB + j * 16 + jl) * KB + (((i * 4 + seg) ^ (jl & (KB / 4 - 1))) << 2);
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

  static_for<0, kCoDepth - 1>([&](auto d) { load(ring[decltype(d)::value]); });
  for (int u0 = 0; u0 < nunits; u0 += kCoDepth) {
    static_for<0, kCoDepth>([&](auto d) {
      constexpr int D = decltype(d)::value;
      load(ring[(D + kCoDepth - 1) % kCoDepth]);
      if (u0 + D < nunits) consume(ring[D]);
    });
  }
  __syncthreads();

  // ---- phase 2: output transform of TB x KB items ---------------------------------------
  constexpr int64_t IN_MAX = (sizeof(MT) == 1 ? 127 : 255) << (PP ? kMaxMShift : 0);
  // ReLU as a lower bound (none: below every value).  A float is bounded through its bit
  // pattern: negative values are negative integers, so one integer maximum with 0 clears
  // them (and -0.0), with INT_MIN it changes nothing.
  const int lo_f = relu ? 0 : (int)0x80000000;
  const int lo_i = relu ? 0 : -128;
#pragma unroll 1
  for (int it = 0; it < (tid < NT2 ? TB * KB / NT2 : 0); ++it) {
    const int item = it * NT2 + tid;
    const int tl = item / KB, kl = item - tl * KB;
    const int k = k0 + kl;
    const int4 ti = s_tile[tl];
    if (!ti.w || k >= g.K) continue;
    const int ty_m = ti.y, tx_m = ti.z;
    const int ksw = ((((kl >> 2) ^ (tl & (KB / 4 - 1))) << 2) | (kl & 3));   // see the store above
    int mi[n][n];
    static_for<0, n>([&](auto i) {
      static_for<0, n>([&](auto j) {
        constexpr int P = decltype(i)::value * n + decltype(j)::value;
        mi[i][j] = (int)M_s[(P * TB + tl) * KB + ksw];
        if constexpr (PP) mi[i][j] <<= sh.template at<P>();
      });
    });
    constexpr int YB = OUT == 0 ? 4 : 1;             // bytes of one output
    char* yitem = static_cast<char*>(yv) + ((((long)ti.x * g.H + ty_m) * g.W + tx_m) * g.K + k) * YB;
    const long wkb = (long)g.W * g.K * YB, kb1 = (long)g.K * YB;
    // FULL: no lane of the wave has a tile that reaches past the image (always so when the
    // tile edge divides H and W): the stores need no edge tests
    auto finish = [&]<const IMat& FT, int64_t FIN, bool FULL>(auto& num) {
      static_for<0, M>([&](auto i) {
        static_for<0, M>([&](auto j) {
          constexpr int I = decltype(i)::value, J = decltype(j)::value;
          constexpr int at_mult = shared_mult_index<FT, I, J>();   // one scale for y
          if (FULL || (ty_m + I < g.H && tx_m + J < g.W)) {
            char* at = yitem + (I * wkb + J * kb1);
            if constexpr (OUT == 0) {
              const float v = to_float_approx(entry<FT, FIN, I, J>(num[i][j])) * mu.outer.v[at_mult];
              __builtin_nontemporal_store(max(__float_as_int(v), lo_f), reinterpret_cast<int*>(at));
            } else {
              const int v = cast_code((float)entry<FT, FIN, I, J>(num[i][j]), mu.outer.v[at_mult], 127.f);
              __builtin_nontemporal_store((int8_t)max(v, lo_i), reinterpret_cast<int8_t*>(at));
            }
          }
        });
      });
    };
    const bool inside = ty_m + M <= g.H && tx_m + M <= g.W;
    const bool all_inside = __builtin_amdgcn_ballot_w64(!inside) == 0;
    if constexpr (LEG) {
      acc_t<TBL::PinvT, IN_MAX> num1[n][n];
      sandwich<TBL::PinvT, IN_MAX>(mi, num1);
      uint32_t m1[n][n];
      cast_result_biased<TBL::PinvT, IN_MAX, true>(num1, mu.inner, 127.f, m1);
      acc_t<TBL::APT, 127> num2[M][M];
      sandwich_codes<TBL::APT, 127>(m1, num2);
      if (all_inside)
        finish.template operator()<TBL::APT, 127, true>(num2);
      else
        finish.template operator()<TBL::APT, 127, false>(num2);
    } else {
      acc_t<TBL::AT, IN_MAX> num[M][M];
      sandwich<TBL::AT, IN_MAX>(mi, num);
      if (all_inside)
        finish.template operator()<TBL::AT, IN_MAX, true>(num);
      else
        finish.template operator()<TBL::AT, IN_MAX, false>(num);
    }
  }
}

template <int M, bool LEG, typename MT, int OUT, bool PP, bool FRAG, int TB, int KB, int NW, int WPE,
          int DEPTH>
static hipError_t conout_launch(const Geometry& g, const int8_t* U, const int8_t* V, void* y,
                                bool relu, const StageMults& mu, const MultTable& mm,
                                const ShiftTable& sh, hipStream_t st) {
  const int tblocks = (g.T + TB - 1) / TB, kblocks = (g.K + KB - 1) / KB;
  const long nblocks = (long)((tblocks + 7) / 8) * 8 * kblocks;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  wino_launch((k_contract_out<M, LEG, MT, OUT, PP, FRAG, TB, KB, NW, WPE, DEPTH>),
              dim3((unsigned)nblocks), dim3(NW * 64), st, U, V, y, g, mu, mm, sh, relu ? 1 : 0,
              tblocks, kblocks);
  return hipGetLastError();
}

template <int M, bool LEG, typename MT, int OUT, bool PP, bool FRAG>
static hipError_t conout_shape(const Geometry& g, const int8_t* U, const int8_t* V, void* y,
                               bool relu, const StageMults& mu, const MultTable& mm,
                               const ShiftTable& sh, hipStream_t st) {
  using S = CoShape<M, MT>;
  return conout_launch<M, LEG, MT, OUT, PP, FRAG, S::TB, S::KB, S::NW, 4, S::DEPTH>(g, U, V, y, relu, mu,
                                                                                    mm, sh, st);
}

template <int M, bool LEG, typename MT>
static hipError_t conout_mt(const Geometry& g, const int8_t* U, const int8_t* V, void* y,
                            int out_type, bool relu, const StageMults& mu, const MultTable& mm,
                            const ShiftTable* sh, hipStream_t st) {
  const ShiftTable none{};
  if (out_type != 0 && out_type != 2) return hipErrorInvalidValue;
#define CO_SH(OUT_, PP_, SH_)                                                                    \
  (g.frag ? conout_shape<M, LEG, MT, OUT_, PP_, true>(g, U, V, y, relu, mu, mm, SH_, st) \
          : conout_shape<M, LEG, MT, OUT_, PP_, false>(g, U, V, y, relu, mu, mm, SH_, st))
  if (sh) return out_type == 0 ? CO_SH(0, true, *sh) : CO_SH(2, true, *sh);
  return out_type == 0 ? CO_SH(0, false, none) : CO_SH(2, false, none);
#undef CO_SH
}

template <int M>
hipError_t PerMCO<M>::run(const Geometry& g, bool leg, const int8_t* U, const int8_t* V, void* y,
                          int m_bits, int out_type, bool relu, const StageMults& mu,
                          const MultTable& mm, const ShiftTable* sh, hipStream_t st) {
  if (m_bits == 8)
    return leg ? conout_mt<M, true, int8_t>(g, U, V, y, out_type, relu, mu, mm, sh, st)
               : conout_mt<M, false, int8_t>(g, U, V, y, out_type, relu, mu, mm, sh, st);
  if (m_bits == 9)
    return leg ? conout_mt<M, true, int16_t>(g, U, V, y, out_type, relu, mu, mm, sh, st)
               : conout_mt<M, false, int16_t>(g, U, V, y, out_type, relu, mu, mm, sh, st);
  return hipErrorInvalidValue;
}

// Work groups the kernel would launch for this geometry (rounded block grid).
template <int M>
long PerMCO<M>::blocks(const Geometry& g, int m_bits) {
  const int TB = m_bits == 8 ? CoShape<M, int8_t>::TB : CoShape<M, int16_t>::TB;
  return (long)((g.T + TB - 1) / TB) * ((g.K + 31) / 32);
}

}  // namespace wino
