// Backward pass of one layer (Winograd-aware training with fixed matrices,
// Sections 2 and 4.2), fp32.  A cast passes its gradient on unchanged
// (straight-through), so every step is the adjoint of the matching step of
// eq. 3 and the base change of eq. 4 cancels (A_P^T P^{-T} = A^T, ...): the
// canonical matrices serve both bases.  The forward pass enters through the
// int8 codes U and V that it contracted, dequantised here by their scales.
//
//   dM[p][t][k]  = (A dY_t A^T)[p]                   k_bwd_dm
//   dU[p][t][c]  = s_v[p] sum_k dM[p][t][k] V[p][k][c]   gemm_body<true>   \ one launch,
//   dV[p][k][c]  = s_u[p] sum_t dM[p][t][k] U[p][t][c]   gemm_body<false>  / k_bwd_gemm_both
//   dx[b][h][w][c] = sum over the <= 4 tiles t covering the pixel of
//                    (B dU_t B^T)[its local position in t]       bwd_dx_body  \ one launch,
//   dw[k][c]     = G^T dV G                          bwd_dw_body  / k_bwd_dx_dw
//
// Layouts as in the forward pass: point-major [n*n][items][channels] for
// everything in the transform domain, NHWC for dy and dx, KCRS for dw.
// The launchers of the flex layer's backward kernels (wino_flex_backward.hpp) and
// the column sums of its matrix gradients are at the end of this file.
#include "wino_kernels.hpp"
#include "wino_real_brackets.hpp"

namespace wino {
namespace {

template <int I>
using ICb = std::integral_constant<int, I>;

// dY -> dM.  One lane per (tile, k); output pixels beyond H x W (partial tiles)
// carry no gradient.
template <int M>
__global__ __launch_bounds__(256) void k_bwd_dm(const float* __restrict__ dy,
                                                float* __restrict__ dM, Geometry g) {
  constexpr int n = M + 2;
  const long total = (long)g.T * g.K;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  if (gid >= total) return;
  const int t = (int)(gid / g.K);
  const int k = (int)(gid - (long)t * g.K);
  const int tx = t % g.TW;
  const int ty = (t / g.TW) % g.TH;
  const int b = t / (g.TW * g.TH);
  float v[M][M];
  rfor<0, M>([&](auto i) {
    rfor<0, M>([&](auto j) {
      const int h = ty * M + decltype(i)::value, w = tx * M + decltype(j)::value;
      v[i][j] = (h < g.H && w < g.W) ? dy[(((long)b * g.H + h) * g.W + w) * g.K + k] : 0.f;
    });
  });
  float out[n][n];
  adjoint_bracket_f<TabF<M>::AT>(v, out);
  rfor<0, n>([&](auto i) {
    rfor<0, n>([&](auto j) {
      dM[(long)(decltype(i)::value * n + decltype(j)::value) * total + gid] = out[i][j];
    });
  });
}

// Entries [A0, A1] x [B0, B1] of B dU B^T for one tile, added to acc[a - A0 + AO][b - B0 + BO]:
//   (B dU B^T)[a][b] = sum_i sum_j BT[i][a] dU[i][j] BT[j][b].
// load(i, j) is called only for the (i, j) that a non-zero coefficient needs.
template <const RMat& BT, int A0, int A1, int B0, int B1, int AO, int BO, int ACC, class Load>
__device__ __forceinline__ void dx_entries(Load&& load, float (&acc)[ACC][ACC]) {
  constexpr int n = BT.rows;
  constexpr auto row_used = [](int i) {
    for (int a = A0; a <= A1; ++a)
      if (BT.a[i][a].num != 0) return true;
    return false;
  };
  constexpr auto col_used = [](int j) {
    for (int b = B0; b <= B1; ++b)
      if (BT.a[j][b].num != 0) return true;
    return false;
  };
  float part[A1 - A0 + 1][n];                    // part[a][j] = sum_i BT[i][a] dU[i][j]
  rfor<0, n>([&](auto j) {
    constexpr int J = decltype(j)::value;
    if constexpr (col_used(J)) {
      rfor<A0, A1 + 1>([&](auto a) { part[decltype(a)::value - A0][J] = 0.f; });
      rfor<0, n>([&](auto i) {
        constexpr int I = decltype(i)::value;
        if constexpr (row_used(I)) {
          const float v = load(i, j);
          rfor<A0, A1 + 1>([&](auto a) {
            constexpr Rat c = BT.a[I][decltype(a)::value];
            if constexpr (c.num != 0)
              part[decltype(a)::value - A0][J] = __builtin_fmaf(
                  (float)((double)c.num / (double)c.den), v, part[decltype(a)::value - A0][J]);
          });
        }
      });
    }
  });
  rfor<A0, A1 + 1>([&](auto a) {
    rfor<B0, B1 + 1>([&](auto b) {
      float sum = 0.f;
      rfor<0, n>([&](auto j) {
        constexpr Rat c = BT.a[decltype(j)::value][decltype(b)::value];
        if constexpr (c.num != 0)
          sum = __builtin_fmaf((float)((double)c.num / (double)c.den),
                               part[decltype(a)::value - A0][decltype(j)::value], sum);
      });
      acc[decltype(a)::value - A0 + AO][decltype(b)::value - B0 + BO] += sum;
    });
  });
}

// dU -> dx.  Tile (ty, tx) reads input rows ty*M - 1 ... ty*M + M (local rows
// 0 ... M + 1), so the M x M pixels starting at (ty*M, tx*M) are its local rows and
// columns 1 ... M, local row M + 1 of the tile above (on the first of them) and
// local row 0 of the tile below (on the last), columns and corners alike.  One
// lane per (tile, channel) gathers those nine contributions for its M x M pixels,
// in a fixed order; no tile ever writes a pixel of another.
template <int M>
__device__ __forceinline__ void bwd_dx_body(const float* __restrict__ dU, float* __restrict__ dx,
                                            const Geometry& g, unsigned block) {
  constexpr int n = M + 2;
  static constexpr RMat BT = TabF<M>::BT;
  const long total = (long)g.T * g.C;
  const long gid = (long)block * 256 + threadIdx.x;
  if (gid >= total) return;
  const int t = (int)(gid / g.C);
  const int c = (int)(gid - (long)t * g.C);
  const int tx = t % g.TW;
  const int ty = (t / g.TW) % g.TH;
  const int b = t / (g.TW * g.TH);
  float acc[M][M];
  rfor<0, M>([&](auto i) { rfor<0, M>([&](auto j) { acc[i][j] = 0.f; }); });
  // neighbour (DY, DX): its local rows [A0, A1] land on my pixel rows AO ...
  auto neighbour = [&](auto dyc, auto dxc) {
    constexpr int DY = decltype(dyc)::value, DX = decltype(dxc)::value;
    constexpr int A0 = DY < 0 ? M + 1 : DY > 0 ? 0 : 1, A1 = DY < 0 ? M + 1 : DY > 0 ? 0 : M;
    constexpr int B0 = DX < 0 ? M + 1 : DX > 0 ? 0 : 1, B1 = DX < 0 ? M + 1 : DX > 0 ? 0 : M;
    constexpr int AO = DY > 0 ? M - 1 : 0, BO = DX > 0 ? M - 1 : 0;
    const int nty = ty + DY, ntx = tx + DX;
    if (nty < 0 || nty >= g.TH || ntx < 0 || ntx >= g.TW) return;
    const float* src = dU + (((long)b * g.TH + nty) * g.TW + ntx) * g.C + c;
    dx_entries<BT, A0, A1, B0, B1, AO, BO>(
        [&](auto i, auto j) { return src[(long)(decltype(i)::value * n + decltype(j)::value) * total]; },
        acc);
  };
  rfor<0, 3>([&](auto dyi) {
    rfor<0, 3>([&](auto dxi) {
      neighbour(ICb<decltype(dyi)::value - 1>{}, ICb<decltype(dxi)::value - 1>{});
    });
  });
  rfor<0, M>([&](auto i) {
    rfor<0, M>([&](auto j) {
      const int h = ty * M + decltype(i)::value, w = tx * M + decltype(j)::value;
      if (h < g.H && w < g.W) dx[(((long)b * g.H + h) * g.W + w) * g.C + c] = acc[i][j];
    });
  });
}

template <int M>
__global__ __launch_bounds__(256) void k_bwd_dx(const float* __restrict__ dU,
                                                float* __restrict__ dx, Geometry g) {
  bwd_dx_body<M>(dU, dx, g, blockIdx.x);
}

// dV -> dw[k][c][3][3].
template <int M>
__device__ __forceinline__ void bwd_dw_body(float* __restrict__ dV, float* __restrict__ dw,
                                            const Geometry& g, unsigned block, int parts) {
  constexpr int n = M + 2;
  const long total = (long)g.K * g.C;
  const long gid = (long)block * 256 + threadIdx.x;
  if (gid >= total) return;
  float v[n][n];
  load_summed_dv<n>(dV, total, gid, parts, true, v);
  float out[3][3];
  adjoint_bracket_f<TabF<M>::G>(v, out);
  rfor<0, 3>([&](auto a) {
    rfor<0, 3>([&](auto bb) {
      dw[gid * 9 + decltype(a)::value * 3 + decltype(bb)::value] = out[a][bb];
    });
  });
}

template <int M>
__global__ __launch_bounds__(256) void k_bwd_dw(float* __restrict__ dV, float* __restrict__ dw,
                                                Geometry g, int parts) {
  bwd_dw_body<M>(dV, dw, g, blockIdx.x, parts);
}

// The last two steps are independent of each other: one launch, the first nb_dw
// work groups transform dV into dw (few, and the longer chain of loads where dV
// comes in parts: they start first), the rest gather dx.
template <int M>
__global__ __launch_bounds__(256, (M <= 4 ? 4 : 2)) void k_bwd_dx_dw(const float* __restrict__ dU,
                                                   float* __restrict__ dx,
                                                   float* __restrict__ dV,
                                                   float* __restrict__ dw, Geometry g,
                                                   unsigned nb_dw, int parts) {
  if (blockIdx.x < nb_dw)
    bwd_dw_body<M>(dV, dw, g, blockIdx.x, parts);
  else
    bwd_dx_body<M>(dU, dx, g, blockIdx.x - nb_dw);
}

// ---------------------------------------------------------------------------
// Contraction gradients: n*n GEMMs  C[p][row][col] = scale[p] * sum_red
// A(p, row, red) * B[p][red][col]  with fp32 A (dM) and int8 B (codes).
//   ARED = true : A is [p][row][red]  (dU: row = t, red = k, col = c, B = V)
//   ARED = false: A is [p][red][row]  (dV: row = k, red = t, col = c, B = U)
// The products run on the bf16 matrix pipe without giving up fp32 accuracy: an
// fp32 value is cut into three bf16 pieces of 8 significant bits each (truncate,
// subtract, truncate, subtract: both subtractions are exact), the int8 codes
// are bf16 values as they stand, so every piece * code product is exact in the
// fp32 accumulator of v_mfma_f32_32x32x16_bf16 and what is lost is what lies
// below the 24th bit of A.  Three such MFMAs do the work of eight fp32 ones in
// 3/16 of their cycles, which leaves LDS traffic and the splitting arithmetic
// as the costs to keep down: hence the large tiles.
// Work group = 4 waves (2 x 2) = (64 MB) x (64 NB) outputs, (32 MB) x (32 NB)
// per wave as MB x NB blocks of 32 x 32, MB and NB 1 or 2.  The reduction runs
// in chunks of 32 staged through LDS with the reduction index contiguous
// ([row][red] and [col][red], rows of 40 bf16 = 80 bytes: 16-byte aligned
// fragments, and the 32 rows a fragment read touches fall on distinct banks),
// the next chunk's global loads in flight during the MFMAs.  Where the
// reduction index is the slow one in memory (B always, A for dV) a lane loads
// the same columns of two consecutive reduction rows and stores the pairs as
// dwords.  red and cols are multiples of 4 resp. 16 (K and C are multiples of
// 16), rows and red are otherwise arbitrary: out-of-range elements are staged
// as zeros, out-of-range outputs are not stored.  Non-finite dM gives NaN.
// ---------------------------------------------------------------------------
using v4f = __attribute__((ext_vector_type(4))) float;
using v2u = __attribute__((ext_vector_type(2))) unsigned;
using v16f = __attribute__((ext_vector_type(16))) float;
using bf16x8 = __attribute__((ext_vector_type(8))) __bf16;

constexpr int kGR = 32;        // reduction chunk
constexpr int kLdH = 40;       // bf16 per staged row: the chunk and 8 of padding
constexpr int kXcds = 8;

struct GemmArgs {
  const float* A;
  const int8_t* B;
  float* C;
  int rows, red, cols;
  int row_blocks, col_blocks, units;
  int blocks;                  // splits * ceil(units / 8) * 8 * col_blocks
  int splits, red_split;       // the reduction is cut into `splits` ranges of red_split (a multiple
                               // of the chunk); range s writes its partial sum to C + s * n*n*rows*cols
  long out_stride;             // n*n * rows * cols
};

// LDS of one work group in floats: three pieces of A and B as bf16, or (afterwards) one
// 32 x (32 NB) output block per wave in rows of 32 NB + 4 floats.
constexpr int gemm_lds(int mb, int nb) {
  const int staged = (3 * mb + nb) * 64 * kLdH / 2, out = 4 * 32 * (32 * nb + 4);
  return staged > out ? staged : out;
}

// x = h + m + l up to the bits below the 24th; each piece sits in the upper half of its word
// (for l the caller drops the lower half).
__device__ __forceinline__ void split3(float x, unsigned& h, unsigned& m, unsigned& l) {
  h = __float_as_uint(x) & 0xffff0000u;
  const float r1 = x - __uint_as_float(h);
  m = __float_as_uint(r1) & 0xffff0000u;
  l = __float_as_uint(r1 - __uint_as_float(m));
}
// Two bf16 (upper halves of a and b) as one dword, a at the lower address.
__device__ __forceinline__ unsigned pack2(unsigned a, unsigned b) {
  return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

template <bool ARED, int MB, int NB>
__device__ __forceinline__ void gemm_body(const GemmArgs& ga, const MultTable& scale,
                                          unsigned block, float* __restrict__ smem) {
  constexpr int TR = 64 * MB, TC = 64 * NB;
  const float* __restrict__ A = ga.A;
  const int8_t* __restrict__ B = ga.B;
  float* __restrict__ Cout = ga.C;
  const int rows = ga.rows, red = ga.red, cols = ga.cols;
  const int row_blocks = ga.row_blocks, col_blocks = ga.col_blocks, units = ga.units;
  unsigned short* Ah = reinterpret_cast<unsigned short*>(smem);
  unsigned short* Am = Ah + TR * kLdH;
  unsigned short* Al = Am + TR * kLdH;
  unsigned short* Bt = Al + TR * kLdH;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per_split = ga.blocks / ga.splits;
  const int split = (int)(block / (unsigned)per_split);
  block -= (unsigned)split * (unsigned)per_split;
  const int r_begin = split * ga.red_split, r_end = min(red, r_begin + ga.red_split);
  Cout += (long)split * ga.out_stride;
  // Consecutive blocks are spread round-robin over the 8 XCDs, so block L runs on
  // XCD L % 8.  The column blocks that share one A panel (point p, row block rb: a
  // "unit") are given to consecutive blocks of ONE XCD, whose L2 then serves the
  // panel to all of them; and every XCD takes a contiguous eighth of the units, i.e.
  // all row blocks of four or five points, so that the codes of a point (the B
  // operand of all its row blocks) are fetched by one XCD, not by all eight.
  const int xcd = block % kXcds, slot = block / kXcds;
  const int unit = xcd * ((units + kXcds - 1) / kXcds) + slot / col_blocks;
  if (unit >= units) return;                     // padding blocks (uniform exit, no barrier yet)
  const int cb = slot % col_blocks;
  const int p = unit / row_blocks, rb = unit - p * row_blocks;
  const int row0 = rb * TR, col0 = cb * TC;
  const float* Ap = A + (long)p * rows * red;
  const int8_t* Bp = B + (long)p * red * cols;
  // Pair mapping: reduction rows 2 * rp and 2 * rp + 1 of the chunk, columns 4 * (pq + 16 j) .. + 3.
  const int rp = tid & 15, pq = tid >> 4;

  v4f ra[2 * MB];
  int rbw[2 * NB];
  auto fetch = [&](int r0) {
#pragma unroll
    for (int it = 0; it < 2 * MB; ++it) {
      v4f v = {0.f, 0.f, 0.f, 0.f};
      if constexpr (ARED) {
        const int idx = tid + it * 256;
        const int row = idx >> 3, q = idx & 7;
        if (row0 + row < rows && r0 + 4 * q < r_end)
          v = *reinterpret_cast<const v4f*>(Ap + (long)(row0 + row) * red + r0 + 4 * q);
      } else {
        const int rr = r0 + 2 * rp + (it & 1), quad = pq + 16 * (it >> 1);
        if (rr < r_end && row0 + 4 * quad < rows)
          v = *reinterpret_cast<const v4f*>(Ap + (long)rr * rows + row0 + 4 * quad);
      }
      ra[it] = v;
    }
#pragma unroll
    for (int it = 0; it < 2 * NB; ++it) {
      const int rr = r0 + 2 * rp + (it & 1), quad = pq + 16 * (it >> 1);
      rbw[it] = 0;
      if (rr < r_end && col0 + 4 * quad < cols)
        rbw[it] = *reinterpret_cast<const int*>(Bp + (long)rr * cols + col0 + 4 * quad);
    }
  };
  auto stage = [&]() {
    if constexpr (ARED) {
#pragma unroll
      for (int it = 0; it < 2 * MB; ++it) {
        const int idx = tid + it * 256;
        const int row = idx >> 3, q = idx & 7;
        unsigned h[4], m[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split3(ra[it][e], h[e], m[e], l[e]);
        const int at = row * kLdH + 4 * q;
        *reinterpret_cast<v2u*>(Ah + at) = v2u{pack2(h[0], h[1]), pack2(h[2], h[3])};
        *reinterpret_cast<v2u*>(Am + at) = v2u{pack2(m[0], m[1]), pack2(m[2], m[3])};
        *reinterpret_cast<v2u*>(Al + at) = v2u{pack2(l[0], l[1]), pack2(l[2], l[3])};
      }
    } else {
#pragma unroll
      for (int j = 0; j < MB; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          unsigned h0, m0, l0, h1, m1, l1;
          split3(ra[2 * j][e], h0, m0, l0);
          split3(ra[2 * j + 1][e], h1, m1, l1);
          const int at = (4 * (pq + 16 * j) + e) * kLdH + 2 * rp;
          *reinterpret_cast<unsigned*>(Ah + at) = pack2(h0, h1);
          *reinterpret_cast<unsigned*>(Am + at) = pack2(m0, m1);
          *reinterpret_cast<unsigned*>(Al + at) = pack2(l0, l1);
        }
    }
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // A code as fp32 has at most 7 significant bits: its upper half is the bf16 value.
        const float f0 = (float)(int8_t)((rbw[2 * j] >> (8 * e)) & 0xff);
        const float f1 = (float)(int8_t)((rbw[2 * j + 1] >> (8 * e)) & 0xff);
        *reinterpret_cast<unsigned*>(Bt + (4 * (pq + 16 * j) + e) * kLdH + 2 * rp) =
            pack2(__float_as_uint(f0), __float_as_uint(f1));
      }
  };

  v16f acc[MB][NB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
  const int wr = (wave >> 1) * 32 * MB, wc = (wave & 1) * 32 * NB;
  const int l32 = lane & 31, lk = lane >> 5;
  // MFMA operands: lane -> row (A) or column (B) lane % 32, reduction indices 8 * (lane / 32) .. + 7.
  const int fa = (wr + l32) * kLdH + 8 * lk, fb = (wc + l32) * kLdH + 8 * lk;

  fetch(r_begin);
  for (int r0 = r_begin; r0 < r_end; r0 += kGR) {
    __syncthreads();                  // the previous chunk's fragment reads are done
    stage();
    __syncthreads();
    if (r0 + kGR < r_end) fetch(r0 + kGR);
#pragma unroll
    for (int kk = 0; kk < kGR; kk += 16) {
      bf16x8 bfrag[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b)
        bfrag[b] = *reinterpret_cast<const bf16x8*>(Bt + fb + b * 32 * kLdH + kk);
#pragma unroll
      for (int a = 0; a < MB; ++a) {
        const int at = fa + a * 32 * kLdH + kk;
        const bf16x8 al = *reinterpret_cast<const bf16x8*>(Al + at);
        const bf16x8 am = *reinterpret_cast<const bf16x8*>(Am + at);
        const bf16x8 ah = *reinterpret_cast<const bf16x8*>(Ah + at);
#pragma unroll
        for (int b = 0; b < NB; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bfrag[b], acc[a][b], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < NB; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bfrag[b], acc[a][b], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < NB; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bfrag[b], acc[a][b], 0, 0, 0);
      }
    }
  }

  // acc[a][b][i] holds output (row = 32 a + (i / 4) * 8 + (lane / 32) * 4 + i % 4,
  // col = 32 b + lane % 32) of the wave's block.  32 rows at a time go through the
  // wave's own part of LDS so that they leave in 16-byte stores, a wave writing
  // full row segments of 128 NB bytes.
  constexpr int kLdC = 32 * NB + 4;
  const float s = scale.v[p];
  float* Cs = smem + wave * 32 * kLdC;
  float* Cp = Cout + (long)p * rows * cols;
#pragma unroll
  for (int a = 0; a < MB; ++a) {
    __syncthreads();                  // the fragments (a = 0) resp. the previous rows have been read
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        Cs[((i >> 2) * 8 + lk * 4 + (i & 3)) * kLdC + 32 * b + l32] = acc[a][b][i] * s;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 4 * NB; ++it) {
      const int idx = lane + it * 64;
      const int r = idx / (8 * NB), q = idx % (8 * NB);
      const int row = row0 + wr + 32 * a + r, col = col0 + wc + 4 * q;
      if (row < rows && col < cols)   // cols is a multiple of 16: a quad is inside or outside
        *reinterpret_cast<v4f*>(Cp + (long)row * cols + col) =
            *reinterpret_cast<const v4f*>(Cs + r * kLdC + 4 * q);
    }
  }
}

// Both contractions in one launch (they only share their input dM): the blocks of
// the dV contraction, whose reduction over the tiles is the longer one, come first,
// the blocks of dU fill the compute units as those drain.  Either may have no
// blocks.  MBV: row blocks per wave of dV's tiles (rows = K); dU's tiles are
// always 128 rows (of tiles) high; NB: column blocks per wave of both (cols = C).
template <int MBV, int NB>
__global__ __launch_bounds__(256) void k_bwd_gemm_both(GemmArgs for_dv, MultTable s_u,
                                                        GemmArgs for_du, MultTable s_v) {
  __shared__ __attribute__((aligned(16))) float smem[gemm_lds(2, NB)];
  if (blockIdx.x < (unsigned)for_dv.blocks)
    gemm_body<false, MBV, NB>(for_dv, s_u, blockIdx.x, smem);
  else
    gemm_body<true, 2, NB>(for_du, s_v, blockIdx.x - (unsigned)for_dv.blocks, smem);
}

inline unsigned blocks256(long items) { return (unsigned)((items + 255) / 256); }

template <int M>
hipError_t bwd_transform(int which, const Geometry& g, const float* in, float* out, hipStream_t st) {
  if (which == 0)
    wino_launch((k_bwd_dm<M>), dim3(blocks256((long)g.T * g.K)), dim3(256), st, in, out, g);
  else
    wino_launch((k_bwd_dx<M>), dim3(blocks256((long)g.T * g.C)), dim3(256), st, in, out, g);
  return hipGetLastError();
}

template <int M>
hipError_t bwd_dw(const Geometry& g, float* dV, float* dw, hipStream_t st) {
  wino_launch((k_bwd_dw<M>), dim3(blocks256((long)g.K * g.C)), dim3(256), st, dV, dw, g,
              backward_dv_reader_parts(g));
  return hipGetLastError();
}

template <int M>
hipError_t bwd_dx_dw(const Geometry& g, const float* dU, float* dx, float* dV, float* dw,
                     hipStream_t st) {
  const unsigned nb_dx = blocks256((long)g.T * g.C), nb_dw = blocks256((long)g.K * g.C);
  wino_launch((k_bwd_dx_dw<M>), dim3(nb_dx + nb_dw), dim3(256), st, dU, dx, dV, dw, g, nb_dw,
              backward_dv_reader_parts(g));
  return hipGetLastError();
}

}  // namespace

// Up to this many partial sums of dV are added by the kernels that read dV (load_summed_dv);
// more are added by k_sum_splits first.
constexpr int kReaderParts = 8;

// dV[i] = sum over s < splits of dV[s * count + i], ascending s, i < count.
__global__ __launch_bounds__(256) void k_sum_splits(float* __restrict__ dV, long count, int splits) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float acc = dV[i];
#pragma unroll 4
  for (int sp = 1; sp < splits; ++sp) acc += dV[(long)sp * count + i];
  dV[i] = acc;
}

hipError_t launch_backward_sum_splits(const Geometry& g, float* dV, hipStream_t st) {
  const int splits = backward_dv_splits(g);
  const long count = (long)(g.m + 2) * (g.m + 2) * g.K * g.C;
  if (splits <= kReaderParts || count == 0) return hipSuccess;   // the readers of dV add those up
  wino_launch(k_sum_splits, dim3(blocks256(count)), dim3(256), st, dV, count, splits);
  return hipGetLastError();
}

hipError_t launch_backward_dx_dw(const Geometry& g, const float* dU, float* dx, float* dV,
                                 float* dw, hipStream_t st) {
  switch (g.m) {
    case 2: return bwd_dx_dw<2>(g, dU, dx, dV, dw, st);
    case 4: return bwd_dx_dw<4>(g, dU, dx, dV, dw, st);
    case 6: return bwd_dx_dw<6>(g, dU, dx, dV, dw, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_backward_transform(int which, const Geometry& g, const float* in, float* out,
                                     hipStream_t st) {
  if (which != 0 && which != 1) return hipErrorInvalidValue;
  const long items = which == 0 ? (long)g.T * g.K : (long)g.T * g.C;
  if (items == 0) return hipSuccess;
  switch (g.m) {
    case 2: return bwd_transform<2>(which, g, in, out, st);
    case 4: return bwd_transform<4>(which, g, in, out, st);
    case 6: return bwd_transform<6>(which, g, in, out, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_backward_dw(const Geometry& g, float* dV, float* dw, hipStream_t st) {
  if ((long)g.K * g.C == 0) return hipSuccess;
  switch (g.m) {
    case 2: return bwd_dw<2>(g, dV, dw, st);
    case 4: return bwd_dw<4>(g, dV, dw, st);
    case 6: return bwd_dw<6>(g, dV, dw, st);
    default: return hipErrorInvalidValue;
  }
}

// Column sums of per-work-group partial sums (rows of 64 floats), for up to three
// arrays in one launch: one work group per column, every lane adds its rows in
// ascending order, then a fixed tree over the 256 lanes.
struct PartialSums {
  const float* part[3];
  float* out[3];
  long rows[3];
  int count[3];
};

__global__ __launch_bounds__(256) void k_sum_partials(PartialSums ps) {
  __shared__ float s_sum[256];
  int v = blockIdx.x, which = 0;
  while (which < 2 && v >= ps.count[which]) v -= ps.count[which++];
  const float* part = ps.part[which];
  const long rows = ps.rows[which];
  float acc = 0.f;
  for (long r = threadIdx.x; r < rows; r += 256) acc += part[r * 64 + v];
  s_sum[threadIdx.x] = acc;
  __syncthreads();
#pragma unroll
  for (int half = 128; half > 0; half >>= 1) {
    if ((int)threadIdx.x < half) s_sum[threadIdx.x] += s_sum[threadIdx.x + half];
    __syncthreads();
  }
  if (threadIdx.x == 0) ps.out[which][v] = s_sum[0];
}

hipError_t launch_sum_partials(const float* const part[3], const long rows[3], const int count[3],
                               float* const out[3], hipStream_t st) {
  PartialSums ps;
  int total = 0;
  for (int i = 0; i < 3; ++i) {
    ps.part[i] = part[i];
    ps.out[i] = out[i];
    ps.rows[i] = rows[i];
    ps.count[i] = count[i];
    total += count[i];
  }
  if (total <= 0) return hipSuccess;
  wino_launch(k_sum_partials, dim3((unsigned)total), dim3(256), st, ps);
  return hipGetLastError();
}

#define WINO_BY_M(CALL)            \
  switch (g.m) {                   \
    case 2: return PerMFlexBwd<2>::CALL; \
    case 4: return PerMFlexBwd<4>::CALL; \
    case 6: return PerMFlexBwd<6>::CALL; \
    default: return hipErrorInvalidValue; \
  }

hipError_t launch_flex_backward_output(const Geometry& g, bool legendre, const void* M_, int m_bits,
                                       const float* dy, float* dM, float* part, const FlexMats& fm,
                                       const StageMults& mu, float s_in, hipStream_t st) {
  WINO_BY_M(output(g, legendre, M_, m_bits, dy, dM, part, fm, mu, s_in, st))
}

hipError_t launch_flex_backward_input_weight(const Geometry& g, bool legendre, const int8_t* x,
                                             const float* dU, float* dXt, float* part_in,
                                             const int8_t* w, float* dV, float* dw,
                                             float* part_w, const FlexMats& fm,
                                             const StageMults& mu, float s_in, float s_w,
                                             hipStream_t st) {
  WINO_BY_M(input_weight(g, legendre, x, dU, dXt, part_in, w, dV, dw, part_w, fm, mu, s_in, s_w, st))
}

hipError_t launch_flex_backward_tile_sum(const Geometry& g, const float* dXt, float* dx,
                                         hipStream_t st) {
  WINO_BY_M(tile_sum(g, dXt, dx, st))
}
#undef WINO_BY_M

// Tile shapes of the two contractions: a wave takes two 32-wide blocks along a dimension that is
// longer than one 64-wide tile, else one.
static int dv_row_blocks(const Geometry& g) { return g.K > 64 ? 2 : 1; }
static int col_blocks_per_wave(const Geometry& g) { return g.C > 64 ? 2 : 1; }

// Parts of dV that the kernel reading dV finds and adds up itself.
int backward_dv_reader_parts(const Geometry& g) {
  const int s = backward_dv_splits(g);
  return s <= kReaderParts ? s : 1;
}

// The dV contraction has few outputs (n*n x K x C) and a long reduction (all tiles): while it
// has fewer tiles than the chip has compute units, the reduction is cut into 2^j ranges that
// run as separate work groups and leave partial sums, added up in ascending order: up to eight
// by the filter bracket that reads dV, more by k_sum_splits before it.  Ranges hold at least
// four chunks; at most 32, and at most 64 MB of partial sums.
int backward_dv_splits(const Geometry& g) {
  const long n2 = (long)(g.m + 2) * (g.m + 2);
  const int tr = 64 * dv_row_blocks(g), tc = 64 * col_blocks_per_wave(g);
  const long tiles = n2 * ((g.K + tr - 1) / tr) * ((g.C + tc - 1) / tc);
  const long chunks = ((long)g.T + kGR - 1) / kGR;
  const long bytes = n2 * g.K * g.C * 4;
  int s = 1;
  while (tiles * s < 256 && (long)s * 2 * 4 <= chunks && s < 32 && (long)s * 2 * bytes <= (64L << 20))
    s *= 2;
  return s;
}

static bool gemm_args(bool for_weights, const Geometry& g, const float* dM, const int8_t* codes,
                      float* out, GemmArgs* ga) {
  const int n2 = (g.m + 2) * (g.m + 2);
  const int tr = for_weights ? 64 * dv_row_blocks(g) : 128, tc = 64 * col_blocks_per_wave(g);
  ga->A = dM;
  ga->B = codes;
  ga->C = out;
  ga->rows = for_weights ? g.K : g.T;
  ga->red = for_weights ? g.T : g.K;
  ga->cols = g.C;
  ga->row_blocks = (ga->rows + tr - 1) / tr;
  ga->col_blocks = (ga->cols + tc - 1) / tc;
  const long units = (long)n2 * ga->row_blocks;
  ga->splits = for_weights ? backward_dv_splits(g) : 1;
  const long chunks = ((long)ga->red + kGR - 1) / kGR;
  ga->red_split = (int)((chunks + ga->splits - 1) / ga->splits) * kGR;
  ga->out_stride = (long)n2 * ga->rows * ga->cols;
  const long blocks = (units + kXcds - 1) / kXcds * kXcds * ga->col_blocks * ga->splits;
  ga->units = (int)units;
  ga->blocks = (int)blocks;                      // no outputs: no blocks
  return blocks <= (1L << 30);
}

static hipError_t launch_gemm_pair(const Geometry& g, const GemmArgs& for_dv, const MultTable& s_u,
                                   const GemmArgs& for_du, const MultTable& s_v, hipStream_t st) {
  const unsigned blocks = (unsigned)for_dv.blocks + (unsigned)for_du.blocks;
  if (blocks == 0) return hipSuccess;
  const dim3 grid(blocks), wg(256);
  if (col_blocks_per_wave(g) == 2) {
    if (dv_row_blocks(g) == 2)
      wino_launch((k_bwd_gemm_both<2, 2>), grid, wg, st, for_dv, s_u, for_du, s_v);
    else
      wino_launch((k_bwd_gemm_both<1, 2>), grid, wg, st, for_dv, s_u, for_du, s_v);
  } else {
    if (dv_row_blocks(g) == 2)
      wino_launch((k_bwd_gemm_both<2, 1>), grid, wg, st, for_dv, s_u, for_du, s_v);
    else
      wino_launch((k_bwd_gemm_both<1, 1>), grid, wg, st, for_dv, s_u, for_du, s_v);
  }
  return hipGetLastError();
}

static GemmArgs no_gemm() {
  GemmArgs ga{};
  ga.splits = 1;
  return ga;
}

hipError_t launch_backward_gemm(bool for_weights, const Geometry& g, const float* dM,
                                const int8_t* codes, float* out, const MultTable& scale,
                                hipStream_t st) {
  GemmArgs ga;
  if (!gemm_args(for_weights, g, dM, codes, out, &ga)) return hipErrorInvalidValue;
  return for_weights ? launch_gemm_pair(g, ga, scale, no_gemm(), scale, st)
                     : launch_gemm_pair(g, no_gemm(), scale, ga, scale, st);
}

hipError_t launch_backward_gemms(const Geometry& g, const float* dM, const int8_t* U,
                                 const int8_t* V, float* dU, float* dV, const MultTable& s_u,
                                 const MultTable& s_v, hipStream_t st) {
  GemmArgs for_dv, for_du;
  if (!gemm_args(true, g, dM, U, dV, &for_dv) || !gemm_args(false, g, dM, V, dU, &for_du))
    return hipErrorInvalidValue;
  if ((long)for_dv.blocks + for_du.blocks > (1L << 30)) {
    hipError_t e = launch_backward_gemm(false, g, dM, V, dU, s_v, st);
    return e == hipSuccess ? launch_backward_gemm(true, g, dM, U, dV, s_u, st) : e;
  }
  return launch_gemm_pair(g, for_dv, s_u, for_du, s_v, st);
}

}  // namespace wino
