// Single-kernel variant for narrow layers (C <= 64): input transform -> per-point
// contraction -> output transform in ONE kernel; the Winograd-domain tensors U and M never
// leave the compute unit.  Only x, V and y touch HBM.
//
// Work group = 8 waves, 16 tiles x KB output channels (KB = 64 for an int8 M, 32 for the
// 9-bit int16 M), all n*n Winograd points:
//   A  eight tiles at a time (one per wave): their n*n pixels x 64 channels are staged in
//      LDS with 16-byte loads (in the part of U_s that is still free), every lane
//      transforms one (tile, channel) item exactly as the input-transform kernel does and
//      drops the n*n codes into LDS as U_s[point][tile][channel];
//   B  wave w takes points w, w+8, ...: for each, one 16x16x64 int8 MFMA per 16 output
//      channels, A operand = V rows (k) straight from global / L2, B operand = the 16
//      tiles of U_s; the result is cast at once and written over that point's own U_s rows
//      as M_s[point][tile][k] (same wave, same bytes: program order suffices), so no
//      accumulator outlives a point;
//   C  every lane runs the output transform of (tile, k) items and stores y.
//
// The input transform is recomputed by each of the K / KB work groups that share a tile
// block, so the variant pays off for K <= 64 (one k block).  Wider layers keep M on chip
// with the two-kernel form of wino_conout.hpp instead.
#include "wino_transforms.hpp"

namespace wino {

constexpr int kFT = 16;          // tiles per work group
constexpr int kFC = 64;          // input channels (the whole reduction)
constexpr int kPt = kFT * kFC;   // bytes of one point's block in LDS: 16 tiles x 64 bytes
constexpr int kFW = 8;           // waves per work group

// Byte offset of (tile, byte) inside a point's 1 KB block.  Rows are 64 bytes
// with no padding; the 16-byte segment index is XOR-ed with bits 1-2 of the
// tile so that the eight 16-byte MFMA-operand reads of a pass (8 consecutive
// tiles, same segment) fall on eight distinct bank groups.  U_s[p] and M_s[p]
// use the same map, so M_s[p] overlays U_s[p] exactly.
__device__ __forceinline__ int sw(int tile, int byte) {
  return tile * kFC + ((((byte >> 4) ^ ((tile >> 1) & 3)) << 4) | (byte & 15));
}

// PP: per-point scales -- the cast of point p uses mm.v[p], and its codes enter
// the output bracket shifted left by entry p of sh (<= kMaxMShift, priced into the
// bounds).  Without PP every entry of mm is the same and sh is not read.
template <int M, bool LEG, typename MT, int OUT, bool PP>
__global__ __launch_bounds__(kFW * 64, 6) void k_fused(const int8_t* __restrict__ x,
                                               const int8_t* __restrict__ V,
                                               void* __restrict__ yv, Geometry g, StageMults in_mu,
                                               StageMults out_mu, MultTable mm, ShiftTable sh,
                                               int relu, int tblocks) {
  constexpr int n = M + 2, n2 = n * n;
  constexpr int KB = sizeof(MT) == 1 ? 64 : 32;      // output channels per work group
  constexpr int NKB = KB / 16;                       // 16-wide MFMA column blocks
  constexpr int NT = kFW * 64;                       // lanes per work group
  constexpr int NPW = (n2 + kFW - 1) / kFW;          // points per wave (the last may be empty)
  static_assert(n2 % 4 == 0 && kFT == 2 * kFW);
  constexpr float QM = sizeof(MT) == 1 ? 127.f : 255.f;
  using TB = Tab<M>;
  // U_s, then M_s: one KiB per point, tile-major.  The pixels of a pass (8 tiles x n*n
  // pixels x 64 bytes = n*n half KiB) are staged in the upper half of every point's KiB,
  // pixel `pix` of the pass's tile `w` at stage_at(pix, w): those halves hold the codes of
  // tiles 8-15, which only the second pass writes, after all its pixels have been read.
  __shared__ __attribute__((aligned(16))) int8_t smem[n2 * kPt];
  auto stage_at = [](int pix, int w) { return pix * kPt + kPt / 2 + w * kFC; };

  // Image and pixel origin of the block's 16 tiles, worked out once and read back from LDS
  // by the staging loop and the output transform: ti = {b, ty*M, tx*M, tile exists}.
  __shared__ int4 s_tile[kFT];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register
  const int tb = blockIdx.x % tblocks, kblk = blockIdx.x / tblocks;
  const int t0 = tb * kFT, k0 = kblk * KB;
  const int jl = lane & 15, seg = lane >> 4;         // MFMA operand row / 16-byte K segment
  if (tid < kFT) {
    const int t = min(t0 + tid, g.T - 1);
    int b, ty, tx;
    tile_coords(g, t, b, ty, tx);
    s_tile[tid] = make_int4(b, ty * M, tx * M, t0 + tid < g.T ? 1 : 0);
  }
  __syncthreads();

  // ---- A: input transform of 16 tiles x 64 channels, one tile per wave and pass ----
#pragma unroll 1
  for (int it = 0; it < kFT / kFW; ++it) {
    // stage the n*n pixels x 64 channels of the pass's 8 tiles with 16-byte loads (zeros
    // outside the image, past the last tile or channel)
    if (it) __syncthreads();                         // the previous pass's pixels are consumed
#pragma unroll
    for (int j = 0; j < (kFW * n2 * 4 + NT - 1) / NT; ++j) {
      const int idx = j * NT + tid;
      if (idx < kFW * n2 * 4) {
        const int tq = idx / (n2 * 4), rem = idx - tq * (n2 * 4);
        const int pix = rem >> 2, sg = rem & 3;
        const int4 ti = s_tile[it * kFW + tq];
        v4i v = {0, 0, 0, 0};
        if (ti.w && sg * 16 < g.C) {
          const int a = pix / n, bb = pix - a * n;
          const int h = ti.y - 1 + a, ww = ti.z - 1 + bb;
          if (h >= 0 && h < g.H && ww >= 0 && ww < g.W)
            v = *reinterpret_cast<const v4i*>(x + (((long)ti.x * g.H + h) * g.W + ww) * g.C + sg * 16);
        }
        *reinterpret_cast<v4i*>(smem + stage_at(pix, tq) + sg * 16) = v;
      }
    }
    __syncthreads();
    const int tl = it * kFW + wave;                  // a wave = one tile, 64 channels
    int xi[n][n];
    static_for<0, n>([&](auto a) {
      static_for<0, n>([&](auto bb) {
        xi[a][bb] = smem[stage_at(decltype(a)::value * n + decltype(bb)::value, wave) + lane];
        asm("" : "+v"(xi[a][bb]));                   // keeps the load a sign-extending byte read
      });
    });
    if (it) __syncthreads();                         // this pass's codes go where its pixels were
    int q[n][n];
    if constexpr (LEG) {
      acc_t<TB::PinvT, 127> num1[n][n];
      sandwich<TB::PinvT, 127>(xi, num1);
      uint32_t x1[n][n];
      cast_result_biased<TB::PinvT, 127, true>(num1, in_mu.inner, 127.f, x1);
      acc_t<TB::BPT, 127> num2[n][n];
      sandwich_codes<TB::BPT, 127>(x1, num2);
      cast_result<TB::BPT, 127, !PP>(num2, in_mu.outer, 127.f, q);
    } else {
      acc_t<TB::BT, 127> num[n][n];
      sandwich<TB::BT, 127>(xi, num);
      cast_result<TB::BT, 127, !PP>(num, in_mu.outer, 127.f, q);
    }
    static_for<0, n>([&](auto i) {
      static_for<0, n>([&](auto j) {
        // a dead item (tile or channel out of range) has all-zero input, hence zero codes
        smem[(decltype(i)::value * n + decltype(j)::value) * kPt + sw(tl, lane)] = (int8_t)q[i][j];
      });
    });
  }
  __syncthreads();

  // ---- B: contraction for the wave's points; cast and park as M_s[p][tile][k] ----
  // D[k = 16 kb + 4 seg + v][tile = jl]
  const bool cok = seg * 16 < g.C;
  unsigned voff[NKB];                                // the lane's V row and channel segment
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
    voff[kb] = (unsigned)(min(k0 + kb * 16 + jl, g.K - 1) * g.C + (cok ? seg * 16 : 0));   // clamp, masked at the store
#pragma clang loop unroll_count(3)
  for (int pi = 0; pi < NPW; ++pi) {
    const int p = pi * kFW + wave;
    if (n2 % kFW != 0 && p >= n2) break;             // wave-uniform: this wave has one point less
    const v4i bu = *reinterpret_cast<const v4i*>(smem + p * kPt + sw(jl, seg * 16));
    v4i a4[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      // a segment past C re-reads segment 0: its U_s codes are zero, whatever V holds
      const v4i av = *reinterpret_cast<const v4i*>(V + (long)p * g.K * g.C + voff[kb]);
      a4[kb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bu, v4i{0, 0, 0, 0}, 0, 0, 0);
    }
    const float m_mult = PP ? mm.v[p] : mm.v[0];     // p is wave-uniform
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      uint32_t q[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) q[v] = cast_biased((float)a4[kb][v], m_mult, QM);
      int8_t* dst = smem + p * kPt + sw(jl, (kb * 16 + 4 * seg) * (int)sizeof(MT));
      if constexpr (sizeof(MT) == 1) {
        const uint32_t lo = __builtin_amdgcn_perm(q[1], q[0], 0x0c0c0400u);
        const uint32_t hi = __builtin_amdgcn_perm(q[3], q[2], 0x04000c0cu);
        *reinterpret_cast<uint32_t*>(dst) = lo | hi;
      } else {
        reinterpret_cast<uint32_t*>(dst)[0] = __builtin_amdgcn_perm(q[1], q[0], 0x05040100u);
        reinterpret_cast<uint32_t*>(dst)[1] = __builtin_amdgcn_perm(q[3], q[2], 0x05040100u);
      }
    }
  }
  __syncthreads();

  // ---- C: output transform of 16 tiles x KB channels ----
  // ReLU as a lower bound (none: below every value).  A float is bounded through its bit
  // pattern: negative values are negative integers, so one integer maximum with 0 clears
  // them (and -0.0), with INT_MIN it changes nothing.
  const int lo_f = relu ? 0 : (int)0x80000000;
  const int lo_i = relu ? 0 : -128;
#pragma unroll 1
  for (int it = 0; it < kFT * KB / NT; ++it) {
    int tl, kl;
    int4 ti;
    if constexpr (KB == 64) {
      // a wave = the 64 output channels of one tile: the tile's coordinates, the edge tests
      // and the tile part of every address stay in scalar registers
      tl = it * (NT / KB) + wave, kl = lane;
      const int4 tv = s_tile[tl];
      ti = make_int4(__builtin_amdgcn_readfirstlane(tv.x), __builtin_amdgcn_readfirstlane(tv.y),
                     __builtin_amdgcn_readfirstlane(tv.z), __builtin_amdgcn_readfirstlane(tv.w));
    } else {
      const int item = it * NT + tid;
      tl = item / KB, kl = item - tl * KB;
      ti = s_tile[tl];
    }
    const int k = k0 + kl;
    if (!ti.w || k >= g.K) continue;
    const int ty_m = ti.y, tx_m = ti.z;              // first output row and column
    int mi[n][n];
    static_for<0, n>([&](auto i) {
      static_for<0, n>([&](auto j) {
        mi[i][j] = (int)*reinterpret_cast<const MT*>(
            smem + (decltype(i)::value * n + decltype(j)::value) * kPt + sw(tl, kl * (int)sizeof(MT)));
        if constexpr (PP) mi[i][j] <<= sh.template at<decltype(i)::value * n + decltype(j)::value>();
      });
    });
    constexpr int YB = OUT == 0 ? 4 : 1;             // bytes of one output
    char* ytile = static_cast<char*>(yv) + (((long)ti.x * g.H + ty_m) * g.W + tx_m) * g.K * YB;
    const long wkb = (long)g.W * g.K * YB, kb1 = (long)g.K * YB;
    unsigned kbyte = (unsigned)k * YB;               // the lane's part of every store address
    auto finish = [&]<const IMat& FT, int64_t FIN>(auto& num) {
      static_for<0, M>([&](auto i) {
        static_for<0, M>([&](auto j) {
          constexpr int I = decltype(i)::value, J = decltype(j)::value;
          constexpr int idx = shared_mult_index<FT, I, J>();
          if (ty_m + I < g.H && tx_m + J < g.W) {
            // the lane's part of the address enters the sum inside this block, so that the store
            // takes the form scalar base + 32-bit lane offset (no vector address arithmetic)
            if constexpr (KB == 64) asm("" : "+v"(kbyte));
            char* at = ytile + (I * wkb + J * kb1) + kbyte;
            if constexpr (OUT == 0) {
              const float v = to_float_approx(entry<FT, FIN, I, J>(num[i][j])) * out_mu.outer.v[idx];
              __builtin_nontemporal_store(max(__float_as_int(v), lo_f), reinterpret_cast<int*>(at));
            } else {
              const int v = cast_code((float)entry<FT, FIN, I, J>(num[i][j]), out_mu.outer.v[idx], 127.f);
              __builtin_nontemporal_store((int8_t)max(v, lo_i), reinterpret_cast<int8_t*>(at));
            }
          }
        });
      });
    };
    constexpr int64_t IN_MAX = (sizeof(MT) == 1 ? 127 : 255) << (PP ? kMaxMShift : 0);
    if constexpr (LEG) {
      acc_t<TB::PinvT, IN_MAX> num1[n][n];
      sandwich<TB::PinvT, IN_MAX>(mi, num1);
      uint32_t m1[n][n];
      cast_result_biased<TB::PinvT, IN_MAX, true>(num1, out_mu.inner, 127.f, m1);
      acc_t<TB::APT, 127> num2[M][M];
      sandwich_codes<TB::APT, 127>(m1, num2);
      finish.template operator()<TB::APT, 127>(num2);
    } else {
      acc_t<TB::AT, IN_MAX> num[M][M];
      sandwich<TB::AT, IN_MAX>(mi, num);
      finish.template operator()<TB::AT, IN_MAX>(num);
    }
  }
}

template <int M, bool LEG, typename MT, bool PP>
static hipError_t fused_mt(const Geometry& g, const int8_t* x, const int8_t* V, void* y, int out_type,
                           bool relu, const StageMults& in_mu, const StageMults& out_mu,
                           const MultTable& mm, const ShiftTable& sh, hipStream_t st) {
  constexpr int KB = sizeof(MT) == 1 ? 64 : 32;
  const int tblocks = (g.T + kFT - 1) / kFT, kblocks = (g.K + KB - 1) / KB;
  dim3 grid((unsigned)(tblocks * kblocks));
  const int r = relu ? 1 : 0;
  // One channel chunk only: wider layers take the two-kernel form (input transform, then
  // contraction + output transform), which does not recompute the input transform per block
  // of output channels.
  if (g.C > kFC) return hipErrorInvalidValue;
  if (out_type == 0)
    wino_launch((k_fused<M, LEG, MT, 0, PP>), grid, dim3(kFW * 64), st, x, V, y, g, in_mu,
                       out_mu, mm, sh, r, tblocks);
  else
    wino_launch((k_fused<M, LEG, MT, 2, PP>), grid, dim3(kFW * 64), st, x, V, y, g, in_mu,
                       out_mu, mm, sh, r, tblocks);
  return hipGetLastError();
}

template <int M, bool LEG>
static hipError_t fused_ml(const Geometry& g, const int8_t* x, const int8_t* V, void* y, int m_bits,
                           int out_type, bool relu, const StageMults& in_mu,
                           const StageMults& out_mu, const MultTable& mm, const ShiftTable* sh,
                           hipStream_t st) {
  const ShiftTable none{};
  if (sh)
    return m_bits == 8
               ? fused_mt<M, LEG, int8_t, true>(g, x, V, y, out_type, relu, in_mu, out_mu, mm, *sh, st)
               : fused_mt<M, LEG, int16_t, true>(g, x, V, y, out_type, relu, in_mu, out_mu, mm, *sh, st);
  return m_bits == 8
             ? fused_mt<M, LEG, int8_t, false>(g, x, V, y, out_type, relu, in_mu, out_mu, mm, none, st)
             : fused_mt<M, LEG, int16_t, false>(g, x, V, y, out_type, relu, in_mu, out_mu, mm, none, st);
}

template <int M>
static hipError_t fused_m(const Geometry& g, bool leg, const int8_t* x, const int8_t* V, void* y,
                          int m_bits, int out_type, bool relu, const StageMults& in_mu,
                          const StageMults& out_mu, const MultTable& mm, const ShiftTable* sh,
                          hipStream_t st) {
  return leg ? fused_ml<M, true>(g, x, V, y, m_bits, out_type, relu, in_mu, out_mu, mm, sh, st)
             : fused_ml<M, false>(g, x, V, y, m_bits, out_type, relu, in_mu, out_mu, mm, sh, st);
}

hipError_t launch_fused(const Geometry& g, bool legendre_inner, const int8_t* x, const int8_t* V,
                        void* y, int m_bits, int out_type, bool relu, const StageMults& in_mu,
                        const StageMults& out_mu, const MultTable& mm, const ShiftTable* sh,
                        hipStream_t st) {
  if ((long)g.T * g.K == 0) return hipSuccess;
  if ((m_bits != 8 && m_bits != 9) || (out_type != 0 && out_type != 2)) return hipErrorInvalidValue;
  switch (g.m) {
    case 2: return fused_m<2>(g, legendre_inner, x, V, y, m_bits, out_type, relu, in_mu, out_mu, mm, sh, st);
    case 4: return fused_m<4>(g, legendre_inner, x, V, y, m_bits, out_type, relu, in_mu, out_mu, mm, sh, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace wino
