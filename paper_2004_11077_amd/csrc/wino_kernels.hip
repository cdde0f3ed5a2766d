// Contraction kernel (gfx950 int8 MFMA) and the per-stage dispatchers.
#include "wino_kernels.hpp"

namespace wino {


typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Pending event pairs of this thread, oldest first; every launch takes one.
constexpr int kMaxPendingProfiles = 8;
static thread_local ProfileEvents t_profile[kMaxPendingProfiles];
static thread_local int t_profile_count = 0;

void set_profile_events(hipEvent_t start, hipEvent_t stop) {
  if (t_profile_count == kMaxPendingProfiles) --t_profile_count;   // full: replace the newest
  t_profile[t_profile_count++] = ProfileEvents{start, stop};
}

ProfileEvents take_profile_events() {
  if (t_profile_count == 0) return ProfileEvents{nullptr, nullptr};
  const ProfileEvents p = t_profile[0];
  for (int i = 1; i < t_profile_count; ++i) t_profile[i - 1] = t_profile[i];
  --t_profile_count;
  return p;
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
constexpr int kKT = 128;

// One cast kept in its biased float form: the code sits, in two's complement,
// in the low bits of the returned pattern (0x4B400000 + q), so packing needs
// only the low byte (or half) of each value.
__device__ __forceinline__ uint32_t cast_biased(float v, float mult, float qmax) {
  constexpr float kMagic = 12582912.0f;
  float t = __builtin_fmaf(v, mult, kMagic);
  t = __builtin_amdgcn_fmed3f(t, kMagic - qmax, kMagic + qmax);
  return __float_as_uint(t);
}

// kTT: tile rows (t) per work group, 128 or 64 (small problems: twice the work groups).
template <typename MT, int kCK, int kTT>
__global__ __launch_bounds__(256) void k_contract(const int8_t* __restrict__ U,
                                                  const int8_t* __restrict__ V,
                                                  MT* __restrict__ Mo, int T, int C, int K,
                                                  int tblocks, int kblocks, int tgroups, int tpg,
                                                  int units, MultTable mults, float qmax) {
  constexpr int kRow = kCK + 16;               // padded LDS row
  constexpr int LPR = kCK / 16;                // lanes per staged row
  constexpr int RPP = 256 / LPR;               // rows staged per pass
  constexpr int NPA = kKT / RPP;               // staging passes for V
  constexpr int NPB = kTT / RPP;               // staging passes for U
  constexpr int JT = kTT / 64;                 // 32-wide t blocks per wave
  constexpr int kSm = (kKT + kTT) * kRow;      // also holds the [t][k] output block
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
  const float mult = mults.v[p];               // cast multiplier of this point (uniform)

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wt = wave & 1, wk = wave >> 1;
  const int r = lane & 31, h = lane >> 5;

  // Addresses are a block-uniform 64-bit base (scalar registers) plus a 32-bit
  // lane offset (the host keeps 128 * C and 128 * K below 2^31).
  const int8_t* Vp = V + ((long)p * K + k0) * C;
  const int8_t* Up = U + ((long)p * T + t0) * C;
  MT* Mp = Mo + ((long)p * T + t0) * K + k0;
  const int krows = K - k0, trows = T - t0;      // rows of this block that exist (>= 1)

  // staging map: LPR lanes cover one row chunk; rows past the edge are read
  // from the last existing row (their products land in outputs never stored)
  const int srow = tid / LPR, sseg = (tid % LPR) * 16;
  uint32_t oa[NPA], ob[NPB];
#pragma unroll
  for (int i = 0; i < NPA; ++i)
    oa[i] = (uint32_t)min(srow + i * RPP, krows - 1) * (uint32_t)C + sseg;
#pragma unroll
  for (int i = 0; i < NPB; ++i)
    ob[i] = (uint32_t)min(srow + i * RPP, trows - 1) * (uint32_t)C + sseg;
  // one register set: the next chunk is in flight while this one feeds the MFMAs
  // (a second set costs a third of the occupancy and measured slower)
  v4i ra[NPA], rb[NPB];
  auto fetch = [&](int c0) {
    if (c0 + kCK <= C) {               // uniform: the whole chunk lies inside C
#pragma unroll
      for (int i = 0; i < NPA; ++i) ra[i] = *reinterpret_cast<const v4i*>(Vp + c0 + oa[i]);
#pragma unroll
      for (int i = 0; i < NPB; ++i) rb[i] = *reinterpret_cast<const v4i*>(Up + c0 + ob[i]);
    } else {
      // last chunk when C is not a multiple of the chunk: columns past C are
      // read from a clamped in-bounds column and zeroed, without branching
      const bool ok = c0 + sseg < C;
      const int cc = ok ? c0 : C - 16 - sseg;
      const int keep = ok ? -1 : 0;
#pragma unroll
      for (int i = 0; i < NPA; ++i) ra[i] = *reinterpret_cast<const v4i*>(Vp + cc + oa[i]) & keep;
#pragma unroll
      for (int i = 0; i < NPB; ++i) rb[i] = *reinterpret_cast<const v4i*>(Up + cc + ob[i]) & keep;
    }
  };

  v16i acc[2][JT];
  // FIRST: the accumulators start from the constant zero operand of the first
  // MFMA instead of being cleared beforehand.
  auto chunk = [&]<bool FIRST>(int c0) {
    if constexpr (!FIRST) __syncthreads();   // previous chunk fully consumed
#pragma unroll
    for (int i = 0; i < NPA; ++i) *reinterpret_cast<v4i*>(sA + (srow + i * RPP) * kRow + sseg) = ra[i];
#pragma unroll
    for (int i = 0; i < NPB; ++i) *reinterpret_cast<v4i*>(sB + (srow + i * RPP) * kRow + sseg) = rb[i];
    __syncthreads();
    if (c0 + kCK < C) fetch(c0 + kCK);
#pragma unroll
    for (int ks = 0; ks < kCK / 32; ++ks) {
      v4i fa[2], fb[JT];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const v4i*>(sA + (wk * 64 + i * 32 + r) * kRow + ks * 32 + h * 16);
#pragma unroll
      for (int j = 0; j < JT; ++j)
        fb[j] = *reinterpret_cast<const v4i*>(sB + (wt * (kTT / 2) + j * 32 + r) * kRow + ks * 32 + h * 16);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < JT; ++j) {
          if (FIRST && ks == 0)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], v16i{}, 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
  };

  fetch(0);
  chunk.template operator()<true>(0);
  for (int c0 = kCK; c0 < C; c0 += kCK) chunk.template operator()<false>(c0);

  // acc[i][j][4*g+v] = D[k = 32 i + 8 g + 4 h + v][t = 32 j + r] within the wave's 64 (k) x kTT/2 (t)
  if constexpr (sizeof(MT) == 1) {
    __syncthreads();                     // LDS is reused as the [t][k] output block
    uint32_t* so = reinterpret_cast<uint32_t*>(smem);
    constexpr int kORow = kKT / 4 + 1;   // dwords per row, +1 against bank conflicts
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          uint32_t q[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) q[v] = cast_biased((float)acc[i][j][4 * gq + v], mult, qmax);
          // low bytes of q0..q3 -> one dword (v_perm_b32: selectors 0-3 take bytes of the
          // second operand, 4-7 of the first, 0x0c gives zero)
          const uint32_t lo = __builtin_amdgcn_perm(q[1], q[0], 0x0c0c0400u);
          const uint32_t hi = __builtin_amdgcn_perm(q[3], q[2], 0x04000c0cu);
          const int tl = wt * (kTT / 2) + j * 32 + r;
          const int kl = wk * 64 + i * 32 + 8 * gq + 4 * h;
          so[tl * kORow + (kl >> 2)] = lo | hi;
        }
    __syncthreads();
    // M is written once and read by the next kernel from other compute units: streaming
    // (nontemporal) stores leave no dirty lines for the end-of-kernel write-back (measured:
    // 1 us per kernel at N = 256, and faster at large batch as well)
    const int kq = tid & 31;             // dword within the 128-byte row
    if (kq * 4 < krows) {
#pragma unroll
      for (int it = 0; it < kTT / 8; ++it) {
        const int tl = it * 8 + (tid >> 5);
        if (tl < trows)
          __builtin_nontemporal_store(so[tl * kORow + kq],
                                      reinterpret_cast<uint32_t*>(Mp + ((uint32_t)tl * (uint32_t)K + kq * 4)));
      }
    }
  } else if constexpr (sizeof(MT) == 2) {
    // 9-bit codes (int16): same route as the int8 codes, through LDS as a [t][k]
    // block of 256-byte rows (+16 B against bank conflicts), stored 16 bytes per lane
    __syncthreads();
    constexpr int kORowB = kKT * 2 + 16;
    static_assert(kTT * kORowB <= kSm);
    static_assert(kTT * (kKT + 4) <= kSm);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          uint32_t q[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) q[v] = cast_biased((float)acc[i][j][4 * gq + v], mult, qmax);
          uint2 pk;                      // low halves of q0, q1 and of q2, q3
          pk.x = __builtin_amdgcn_perm(q[1], q[0], 0x05040100u);
          pk.y = __builtin_amdgcn_perm(q[3], q[2], 0x05040100u);
          const int tl = wt * (kTT / 2) + j * 32 + r;
          const int kl = wk * 64 + i * 32 + 8 * gq + 4 * h;
          *reinterpret_cast<uint2*>(smem + tl * kORowB + kl * 2) = pk;
        }
    __syncthreads();
    const int kseg = tid & 15;           // 16-byte segment (8 codes) within the 256-byte row
    if (kseg * 8 < krows) {
#pragma unroll
      for (int it = 0; it < kTT / 16; ++it) {
        const int tl = it * 16 + (tid >> 4);
        if (tl < trows)
          __builtin_nontemporal_store(*reinterpret_cast<const v4i*>(smem + tl * kORowB + kseg * 16),
                                      reinterpret_cast<v4i*>(Mp + ((uint32_t)tl * (uint32_t)K + kseg * 8)));
      }
    }
  } else {
    // unquantised int32 result (calibration, bits_hadamard = 32): stored from registers
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < JT; ++j) {
        const int tl = wt * (kTT / 2) + j * 32 + r;
        if (tl >= trows) continue;
        MT* mrow = Mp + (uint32_t)tl * (uint32_t)K;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int kl = wk * 64 + i * 32 + 8 * gq + 4 * h;
          if (kl >= krows) continue;
          *reinterpret_cast<int4*>(mrow + kl) = make_int4(acc[i][j][4 * gq], acc[i][j][4 * gq + 1],
                                                           acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]);
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

__global__ __launch_bounds__(256) void k_probe_mfma_bf16(int iters, int* __restrict__ sink) {
  using v16f = __attribute__((ext_vector_type(16))) float;
  using bf16x8 = __attribute__((ext_vector_type(8))) __bf16;
  using v4u = __attribute__((ext_vector_type(4))) unsigned;
  // bf16 pairs 1.0 | 0.5 resp. 2.0 | -1.0 (plus a lane-dependent low mantissa bit)
  const unsigned ua = 0x3f803f00u | (threadIdx.x & 1), ub = 0x4000bf80u | ((threadIdx.x >> 1) & 1);
  const v4u wa = {ua, ua, ua, ua}, wb = {ub, ub, ub, ub};
  const bf16x8 a = __builtin_bit_cast(bf16x8, wa), b = __builtin_bit_cast(bf16x8, wb);
  v16f acc[4] = {};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int k = 0; k < 4; ++k)
      acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += acc[k][e];
  if (sum == 12345.678f) sink[0] = 1;        // keeps the loop alive; practically never true
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
  else if (kind == 2)
    wino_launch(k_probe_mfma_bf16, dim3((unsigned)blocks), dim3(256), st, iters, sink);
  else
    wino_launch(k_probe_valu_mad24, dim3((unsigned)blocks), dim3(256), st, iters, 3, sink);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_absmax_i32(const int32_t* __restrict__ v, long count,
                                                    unsigned long long* __restrict__ amax) {
  const int32_t* seg = v + (long)blockIdx.y * count;
  unsigned int m = 0;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long)gridDim.x * 256) {
    const int x = seg[i];
    const unsigned int a = x < 0 ? (unsigned int)(-(long)x) : (unsigned int)x;
    m = a > m ? a : m;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned int o = __shfl_xor(m, off);
    m = o > m ? o : m;
  }
  if ((threadIdx.x & 63) == 0 && m != 0) atomicMax(amax + blockIdx.y, (unsigned long long)m);
}

hipError_t launch_absmax_i32(const int32_t* v, long count, int segments,
                             unsigned long long* amax, hipStream_t st) {
  if (count == 0 || segments == 0) return hipSuccess;
  long nb = (count + 255) / 256;
  if (nb > 256) nb = 256;     // one atomic per wave: keep each target uncontended
  wino_launch(k_absmax_i32, dim3((unsigned)nb, (unsigned)segments), dim3(256), st, v, count, amax);
  return hipGetLastError();
}

hipError_t launch_calibrate_stage(int stage, const Geometry& g, bool leg, int phase,
                                  const void* in, int m_bits, unsigned long long* amax,
                                  const StageMults& mu, bool relu, const ShiftTable* sh,
                                  hipStream_t st) {
#define WINO_CAL_M(MM)                                                                          \
  case MM:                                                                                      \
    return stage == 0   ? PerMCal<MM>::weight(g, leg, phase, (const int8_t*)in, amax, mu, st)   \
           : stage == 1 ? PerMCal<MM>::input(g, leg, phase, (const int8_t*)in, amax, mu, st)    \
                        : PerMCal<MM>::output(g, leg, phase, in, m_bits, amax, mu, relu, sh, st);
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

hipError_t launch_flex_operands(const Geometry& g, bool leg, const int8_t* x, int8_t* U,
                                const int8_t* w, int8_t* V, const FlexMats& fm,
                                const StageMults& mu_in, float mult_u, const StageMults& mu_w,
                                float mult_first, hipStream_t st) {
  switch (g.m) {
    case 2: return PerMFlex<2>::operands(g, leg, x, U, w, V, fm, mu_in, mult_u, mu_w, mult_first, st);
    case 4: return PerMFlex<4>::operands(g, leg, x, U, w, V, fm, mu_in, mult_u, mu_w, mult_first, st);
    case 6: return PerMFlex<6>::operands(g, leg, x, U, w, V, fm, mu_in, mult_u, mu_w, mult_first, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_weight_transform(const Geometry& g, int leg, const int8_t* w, int8_t* V,
                                   const StageMults& mu, hipStream_t st) {
  if ((long)g.K * g.C == 0) return hipSuccess;
  switch (g.m) {
    case 2: return PerM<2>::weight(g, leg, w, V, mu, st);
    case 4: return PerM<4>::weight(g, leg, w, V, mu, st);
    case 6: return PerM<6>::weight(g, leg, w, V, mu, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_input_transform(const Geometry& g, int leg, const int8_t* x, int8_t* U,
                                  const StageMults& mu, hipStream_t st) {
  if ((long)g.T * g.C == 0) return hipSuccess;
  switch (g.m) {
    case 2: return PerM<2>::input(g, leg, x, U, mu, st);
    case 4: return PerM<4>::input(g, leg, x, U, mu, st);
    case 6: return PerM<6>::input(g, leg, x, U, mu, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_operand_transforms(const Geometry& g, int leg, const int8_t* x, int8_t* U,
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

template <int kTT>
static hipError_t contract_tt(const Geometry& g, const int8_t* U, const int8_t* V, void* Mo,
                              int m_bits, const MultTable& mult, hipStream_t st) {
  const int n = g.m + 2;
  const int tblocks = (g.T + kTT - 1) / kTT, kblocks = (g.K + kKT - 1) / kKT;
  const int tgroups = contract_tile_groups(g, kTT);
  const int tpg = (tblocks + tgroups - 1) / tgroups;
  const int units = n * n * tgroups;
  const long nblocks = (long)((units + 7) / 8) * 8 * tpg * kblocks;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  dim3 grid((unsigned)nblocks);
  if (m_bits == 8)
    wino_launch((k_contract<int8_t, 128, kTT>), grid, dim3(256), st, U, V, (int8_t*)Mo, g.T, g.C,
                       g.K, tblocks, kblocks, tgroups, tpg, units, mult, 127.f);
  else if (m_bits == 9)
    wino_launch((k_contract<int16_t, 128, kTT>), grid, dim3(256), st, U, V, (int16_t*)Mo, g.T,
                       g.C, g.K, tblocks, kblocks, tgroups, tpg, units, mult, 255.f);
  else
    wino_launch((k_contract<int32_t, 128, kTT>), grid, dim3(256), st, U, V, (int32_t*)Mo, g.T,
                       g.C, g.K, tblocks, kblocks, tgroups, tpg, units, mult, 0.f);
  return hipGetLastError();
}

// Zero fill in 16-byte stores (a kernel, not hipMemsetAsync, so that a caller may
// capture the launch in a HIP graph).
__global__ __launch_bounds__(256) void k_fill_zero16(v4i* __restrict__ dst, long count16) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < count16; i += (long)gridDim.x * 256)
    dst[i] = v4i{0, 0, 0, 0};
}

hipError_t launch_fill_zero(void* dst, long bytes, hipStream_t st) {
  const long count16 = bytes / 16;
  if (count16 == 0) return hipSuccess;
  long nb = (count16 + 255) / 256;
  if (nb > 4096) nb = 4096;
  wino_launch(k_fill_zero16, dim3((unsigned)nb), dim3(256), st, (v4i*)dst, count16);
  return hipGetLastError();
}

hipError_t launch_contract_output(const Geometry& g, bool leg, const int8_t* U, const int8_t* V,
                                  void* y, int m_bits, int out_type, bool relu,
                                  const StageMults& out_mu, const MultTable& mm,
                                  const ShiftTable* sh, hipStream_t st) {
  if ((long)g.T * g.K == 0) return hipSuccess;
  if (g.C == 0)   // an empty channel sum: y = 0 (K is a multiple of 16, so the size is one of 16 bytes)
    return launch_fill_zero(y, (long)g.N * g.H * g.W * g.K * (out_type == 0 ? 4 : 1), st);
  switch (g.m) {
    case 2: return PerMCO<2>::run(g, leg, U, V, y, m_bits, out_type, relu, out_mu, mm, sh, st);
    case 4: return PerMCO<4>::run(g, leg, U, V, y, m_bits, out_type, relu, out_mu, mm, sh, st);
    case 6: return PerMCO<6>::run(g, leg, U, V, y, m_bits, out_type, relu, out_mu, mm, sh, st);
  }
  return hipErrorInvalidValue;
}

long contract_output_blocks(const Geometry& g, int m_bits) {
  switch (g.m) {
    case 2: return PerMCO<2>::blocks(g, m_bits);
    case 4: return PerMCO<4>::blocks(g, m_bits);
    case 6: return PerMCO<6>::blocks(g, m_bits);
  }
  return 0;
}

hipError_t launch_contract(const Geometry& g, const int8_t* U, const int8_t* V, void* Mo,
                           int m_bits, const MultTable& mult, hipStream_t st) {
  if ((long)g.T * g.K == 0) return hipSuccess;
  if (g.C == 0) {
    // An empty channel sum: every M is the zero code.  k_contract is not launched (its
    // staging loads assume at least one 16-byte channel segment per row).
    const int n0 = g.m + 2;   // K is a multiple of 16, so the byte count is one of 16
    return launch_fill_zero(Mo, (long)n0 * n0 * g.T * g.K * (m_bits == 8 ? 1 : m_bits == 9 ? 2 : 4), st);
  }
  return contract_tile_rows(g) == 64 ? contract_tt<64>(g, U, V, Mo, m_bits, mult, st)
                                     : contract_tt<128>(g, U, V, Mo, m_bits, mult, st);
}

hipError_t launch_output_transform(const Geometry& g, int leg, const void* Mq, int m_bits,
                                   void* y, int out_type, bool relu, const StageMults& mu,
                                   const ShiftTable* sh, hipStream_t st) {
  if ((long)g.T * g.K == 0) return hipSuccess;
  switch (g.m) {
    case 2: return PerM<2>::output(g, leg, Mq, m_bits, y, out_type, relu, mu, sh, st);
    case 4: return PerM<4>::output(g, leg, Mq, m_bits, y, out_type, relu, mu, sh, st);
    case 6: return PerM<6>::output(g, leg, Mq, m_bits, y, out_type, relu, mu, sh, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace wino
