// Contraction kernel (gfx950 int8 MFMA) and the per-stage dispatchers.
#include "wino_kernels.hpp"

namespace wino {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

static thread_local ProfileEvents t_profile = {nullptr, nullptr};

void set_profile_events(hipEvent_t start, hipEvent_t stop) { t_profile = ProfileEvents{start, stop}; }

ProfileEvents take_profile_events() {
  const ProfileEvents p = t_profile;
  t_profile = ProfileEvents{nullptr, nullptr};
  return p;
}

// One symmetric cast: q = clamp(rint(v * mult), +-qmax) with the exact product
// rounded once, ties to even (fma onto 1.5 * 2^23, clamp of the biased float).
__device__ __forceinline__ int cast_code(float v, float mult, float qmax) {
  constexpr float kMagic = 12582912.0f;
  float t = __builtin_fmaf(v, mult, kMagic);
  t = __builtin_amdgcn_fmed3f(t, kMagic - qmax, kMagic + qmax);
  return __float_as_int(t) - 0x4B400000;
}

// ---------------------------------------------------------------------------
// Contraction: per Winograd point p, M[p][t][k] = sum_c U[p][t][c] V[p][k][c],
// a batch of n*n int8 GEMMs (the only dense contraction of the path, hence
// the only MFMA user).
//
// Work group = 4 waves, output block 128 (t) x 128 (k); the channel dimension
// is consumed in chunks of 128 bytes staged through LDS (rows padded by 16 B:
// eight consecutive rows then cover all banks for the 16-byte fragment reads),
// with the next chunk prefetched into registers while the current one feeds
// the MFMAs.  Each wave owns 64 x 64 outputs as 2 x 2 blocks of the 32x32x32
// int8 MFMA.  The A operand is V (rows k), the B operand U (rows t), so a lane
// ends up with four consecutive k of one tile per accumulator quad.
// int8 results are transposed through LDS so that global stores are full
// 128-byte rows; the wider int16 / int32 results are stored from registers.
//
// Blocks are numbered so that all blocks of a (point, group of t blocks) run
// on the same XCD (consecutive work group ids go round-robin over the 8 XCDs,
// each with a private L2): the k blocks that share a set of U rows then share
// one L2, and the number of groups is chosen to spread n*n points evenly.
// ---------------------------------------------------------------------------
constexpr int kTT = 128, kKT = 128;

template <typename MT, int kCK>
__global__ __launch_bounds__(256) void k_contract(const int8_t* __restrict__ U,
                                                  const int8_t* __restrict__ V,
                                                  MT* __restrict__ Mo, int T, int C, int K,
                                                  int tblocks, int kblocks, int tgroups, int tpg,
                                                  int units, float mult, float qmax) {
  constexpr int kRow = kCK + 16;               // padded LDS row
  constexpr int LPR = kCK / 16;                // lanes per staged row
  constexpr int RPP = 256 / LPR;               // rows staged per pass
  constexpr int NP = 128 / RPP;                // passes per operand
  constexpr int kSm = (kKT + kTT) * kRow > kTT * (kKT + 4) ? (kKT + kTT) * kRow : kTT * (kKT + 4);
  __shared__ __attribute__((aligned(16))) int8_t smem[kSm];
  int8_t* sA = smem;                  // V rows (k)
  int8_t* sB = smem + kKT * kRow;     // U rows (t)

  // unit = (point, group of t blocks); all k blocks of a t block are adjacent
  // slots of the same XCD, so U rows are fetched into that L2 once.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int nbu = tpg * kblocks;                 // blocks per unit
  const int unit = (slot / nbu) * 8 + xcd;
  if (unit >= units) return;
  const int inner = slot % nbu;
  const int kb = inner % kblocks;
  const int p = unit / tgroups;
  const int tb = (unit - p * tgroups) * tpg + inner / kblocks;
  if (tb >= tblocks) return;
  const int t0 = tb * kTT, k0 = kb * kKT;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wt = wave & 1, wk = wave >> 1;
  const int r = lane & 31, h = lane >> 5;

  // staging map: 8 lanes cover one 128-byte row chunk, 4 rows per 32 lanes
  const int srow = tid / LPR, sseg = (tid % LPR) * 16;
  const int8_t* ga[NP];
  const int8_t* gb[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int row = srow + i * RPP;
    const int kr = min(k0 + row, K - 1), tr = min(t0 + row, T - 1);   // clamp, mask later
    ga[i] = V + ((long)p * K + kr) * C + sseg;
    gb[i] = U + ((long)p * T + tr) * C + sseg;
  }
  // one register set: the next chunk is in flight while this one feeds the MFMAs
  // (a second set costs a third of the occupancy and measured slower)
  v4i ra0[NP], rb0[NP];
  auto fetch = [&](v4i (&ra)[NP], v4i (&rb)[NP], int c0) {
    // columns past C (last chunk when C is not a multiple of 128) are read
    // from a clamped in-bounds column and zeroed, without branching
    const bool ok = c0 + sseg < C;
    const int cc = ok ? c0 : C - 16 - sseg;
    const int keep = ok ? -1 : 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      ra[i] = *reinterpret_cast<const v4i*>(ga[i] + cc) & keep;
      rb[i] = *reinterpret_cast<const v4i*>(gb[i] + cc) & keep;
    }
  };

  v16i acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = v16i{};

  auto chunk = [&](v4i (&ra)[NP], v4i (&rb)[NP], int c0) {
    if (c0) __syncthreads();             // previous chunk fully consumed
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      *reinterpret_cast<v4i*>(sA + (srow + i * RPP) * kRow + sseg) = ra[i];
      *reinterpret_cast<v4i*>(sB + (srow + i * RPP) * kRow + sseg) = rb[i];
    }
    __syncthreads();
    if (c0 + kCK < C) fetch(ra, rb, c0 + kCK);
#pragma unroll
    for (int ks = 0; ks < kCK / 32; ++ks) {
      v4i fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const v4i*>(sA + (wk * 64 + i * 32 + r) * kRow + ks * 32 + h * 16);
        fb[i] = *reinterpret_cast<const v4i*>(sB + (wt * 64 + i * 32 + r) * kRow + ks * 32 + h * 16);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  fetch(ra0, rb0, 0);
  for (int c0 = 0; c0 < C; c0 += kCK) chunk(ra0, rb0, c0);

  // acc[i][j][4*g+v] = D[k = 32 i + 8 g + 4 h + v][t = 32 j + r] within the wave's 64 x 64
  if constexpr (sizeof(MT) == 1) {
    __syncthreads();                     // LDS is reused as the [t][k] output block
    uint32_t* so = reinterpret_cast<uint32_t*>(smem);
    constexpr int kORow = kKT / 4 + 1;   // dwords per row, +1 against bank conflicts
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          uint32_t pk = 0;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int q = cast_code((float)acc[i][j][4 * gq + v], mult, qmax);
            pk |= ((uint32_t)q & 0xffu) << (8 * v);
          }
          const int tl = wt * 64 + j * 32 + r;
          const int kl = wk * 64 + i * 32 + 8 * gq + 4 * h;
          so[tl * kORow + (kl >> 2)] = pk;
        }
    __syncthreads();
    const int kq = tid & 31;             // dword within the 128-byte row
    if (k0 + kq * 4 < K) {
#pragma unroll
      for (int it = 0; it < kTT / 8; ++it) {
        const int tl = it * 8 + (tid >> 5);
        if (t0 + tl < T)
          *reinterpret_cast<uint32_t*>(Mo + ((long)p * T + t0 + tl) * K + k0 + kq * 4) =
              so[tl * kORow + kq];
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int t = t0 + wt * 64 + j * 32 + r;
        if (t >= T) continue;
        MT* mrow = Mo + ((long)p * T + t) * K;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int kk = k0 + wk * 64 + i * 32 + 8 * gq + 4 * h;
          if (kk >= K) continue;
          int q[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            if constexpr (sizeof(MT) == 4)
              q[v] = acc[i][j][4 * gq + v];
            else
              q[v] = cast_code((float)acc[i][j][4 * gq + v], mult, qmax);
          }
          if constexpr (sizeof(MT) == 2) {
            uint2 pk;
            pk.x = ((uint32_t)q[0] & 0xffffu) | ((uint32_t)q[1] << 16);
            pk.y = ((uint32_t)q[2] & 0xffffu) | ((uint32_t)q[3] << 16);
            *reinterpret_cast<uint2*>(mrow + kk) = pk;
          } else {
            *reinterpret_cast<int4*>(mrow + kk) = make_int4(q[0], q[1], q[2], q[3]);
          }
        }
      }
  }
}

// ---------------------------------------------------------------------------
// Peak probes (measurement helpers): register-only loops that show what this
// device sustains on the two units the hot path is priced against.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_probe_mfma_i8(int iters, int* __restrict__ sink) {
  const int lane = threadIdx.x;
  v4i a = {lane, lane + 1, lane + 2, lane + 3}, b = {lane ^ 5, lane ^ 9, lane ^ 17, lane ^ 33};
  v16i acc[4] = {};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[k], 0, 0, 0);
  }
  int sum = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int e = 0; e < 16; ++e) sum ^= acc[k][e];
  if (sum == 0x7fffffff) sink[0] = sum;      // keeps the loop alive; practically never true
}

__global__ __launch_bounds__(256) void k_probe_valu_mad24(int iters, int c, int* __restrict__ sink) {
  int acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = threadIdx.x + k;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int k = 0; k < 8; ++k)
      asm volatile("v_mad_i32_i24 %0, %1, %2, %0" : "+v"(acc[k]) : "v"(acc[(k + 1) & 7]), "s"(c));
  }
  int sum = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) sum ^= acc[k];
  if (sum == 0x7fffffff) sink[0] = sum;
}

hipError_t launch_probe(int kind, int blocks, int iters, int* sink, hipStream_t st) {
  if (kind == 0)
    wino_launch(k_probe_mfma_i8, dim3((unsigned)blocks), dim3(256), st, iters, sink);
  else
    wino_launch(k_probe_valu_mad24, dim3((unsigned)blocks), dim3(256), st, iters, 3, sink);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_absmax_i32(const int32_t* __restrict__ v, long count,
                                                    unsigned long long* __restrict__ amax) {
  unsigned int m = 0;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long)gridDim.x * 256) {
    const int x = v[i];
    const unsigned int a = x < 0 ? (unsigned int)(-(long)x) : (unsigned int)x;
    m = a > m ? a : m;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned int o = __shfl_xor(m, off);
    m = o > m ? o : m;
  }
  if ((threadIdx.x & 63) == 0 && m != 0) atomicMax(amax, (unsigned long long)m);
}

hipError_t launch_absmax_i32(const int32_t* v, long count, unsigned long long* amax,
                             hipStream_t st) {
  if (count == 0) return hipSuccess;
  long nb = (count + 255) / 256;
  if (nb > 256) nb = 256;     // one atomic per wave: keep the single target uncontended
  wino_launch(k_absmax_i32, dim3((unsigned)nb), dim3(256), st, v, count, amax);
  return hipGetLastError();
}

hipError_t launch_calibrate_stage(int stage, const Geometry& g, bool leg, int phase,
                                  const void* in, int m_bits, unsigned long long* amax,
                                  const StageMults& mu, bool relu, hipStream_t st) {
#define WINO_CAL_M(MM)                                                                          \
  case MM:                                                                                      \
    return stage == 0   ? PerMCal<MM>::weight(g, leg, phase, (const int8_t*)in, amax, mu, st)   \
           : stage == 1 ? PerMCal<MM>::input(g, leg, phase, (const int8_t*)in, amax, mu, st)    \
                        : PerMCal<MM>::output(g, leg, phase, in, m_bits, amax, mu, relu, st);
  switch (g.m) {
    WINO_CAL_M(2)
    WINO_CAL_M(4)
    WINO_CAL_M(6)
  }
#undef WINO_CAL_M
  return hipErrorInvalidValue;
}

hipError_t launch_flex_stage(int stage, const Geometry& g, bool leg, int mode, const void* in,
                             int m_bits, void* out, int out_type, bool relu,
                             unsigned long long* amax, const FlexMats& fm, const StageMults& mu,
                             float mult, hipStream_t st) {
  const long items = stage == 0 ? (long)g.K * g.C : stage == 1 ? (long)g.T * g.C : (long)g.T * g.K;
  if (items == 0) return hipSuccess;
#define WINO_FLEX_M(MM)                                                                          \
  case MM:                                                                                       \
    return stage == 0   ? PerMFlex<MM>::weight(g, leg, mode, (const int8_t*)in, (int8_t*)out,    \
                                               amax, fm, mu, mult, st)                           \
           : stage == 1 ? PerMFlex<MM>::input(g, leg, mode, (const int8_t*)in, (int8_t*)out,     \
                                              amax, fm, mu, mult, st)                            \
                        : PerMFlex<MM>::output(g, leg, mode, in, m_bits, out, out_type, relu,    \
                                               amax, fm, mu, mult, st);
  switch (g.m) {
    WINO_FLEX_M(2)
    WINO_FLEX_M(4)
    WINO_FLEX_M(6)
  }
#undef WINO_FLEX_M
  return hipErrorInvalidValue;
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

hipError_t launch_operand_transforms(const Geometry& g, bool leg, const int8_t* x, int8_t* U,
                                     const int8_t* w, int8_t* V, const StageMults& mu_in,
                                     const StageMults& mu_w, hipStream_t st) {
  if ((long)g.T * g.C == 0) return launch_weight_transform(g, leg, w, V, mu_w, st);
  if ((long)g.K * g.C == 0) return launch_input_transform(g, leg, x, U, mu_in, st);
  switch (g.m) {
    case 2: return PerM<2>::operands(g, leg, x, U, w, V, mu_in, mu_w, st);
    case 4: return PerM<4>::operands(g, leg, x, U, w, V, mu_in, mu_w, st);
    case 6: return PerM<6>::operands(g, leg, x, U, w, V, mu_in, mu_w, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_contract(const Geometry& g, const int8_t* U, const int8_t* V, void* Mo,
                           int m_bits, float mult, hipStream_t st) {
  if ((long)g.T * g.K == 0) return hipSuccess;
  const int n = g.m + 2;
  const int tblocks = (g.T + kTT - 1) / kTT, kblocks = (g.K + kKT - 1) / kKT;
  int tgroups = 1;                                   // smallest split that fills 8 XCDs evenly
  while (tgroups < 8 && (n * n * tgroups) % 8 != 0 && tgroups * 2 <= tblocks) tgroups *= 2;
  const int tpg = (tblocks + tgroups - 1) / tgroups;
  const int units = n * n * tgroups;
  const long nblocks = (long)((units + 7) / 8) * 8 * tpg * kblocks;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  dim3 grid((unsigned)nblocks);
  if (m_bits == 8)
    wino_launch((k_contract<int8_t, 128>), grid, dim3(256), st, U, V, (int8_t*)Mo, g.T, g.C,
                       g.K, tblocks, kblocks, tgroups, tpg, units, mult, 127.f);
  else if (m_bits == 9)
    wino_launch((k_contract<int16_t, 128>), grid, dim3(256), st, U, V, (int16_t*)Mo, g.T,
                       g.C, g.K, tblocks, kblocks, tgroups, tpg, units, mult, 255.f);
  else
    wino_launch((k_contract<int32_t, 128>), grid, dim3(256), st, U, V, (int32_t*)Mo, g.T,
                       g.C, g.K, tblocks, kblocks, tgroups, tpg, units, mult, 0.f);
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
