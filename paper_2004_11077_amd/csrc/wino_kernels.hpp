// Internal launcher interface between the C ABI (wino_api.cpp) and the HIP
// kernels (wino_kernels.hip).  Not part of the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>

namespace wino {

// Optional per-launch timing: a pair of HIP events handed over with
// set_profile_events() is attached to the NEXT kernel this thread launches
// through wino_launch (the events then carry that dispatch's own begin and
// end timestamps); the pair is consumed by that launch.  Pairs queue up (at
// most 8 pending): the k-th pending pair goes to the k-th launch from now.
struct ProfileEvents {
  hipEvent_t start, stop;
};
void set_profile_events(hipEvent_t start, hipEvent_t stop);
ProfileEvents take_profile_events();

template <class K, class... Args>
inline void wino_launch(K kernel, dim3 grid, dim3 block, hipStream_t st, Args... args) {
  const ProfileEvents p = take_profile_events();
  if (p.start || p.stop)
    hipExtLaunchKernelGGL(kernel, grid, block, 0, st, p.start, p.stop, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

// Records the text of a failure for wino_last_error() on this thread and returns `code`
// (for the parts of the C ABI that live outside wino_api.cpp).
int report_error(int code, const char* fmt, ...);

constexpr int kMaxPts = 64;   // n*n for n = 8

// fp32 multipliers of one cast, indexed [i*cols + j] (Section 4.2 cast after a
// bracket; value = s_prev / (rho_i rho_j s_next), rounded to fp32 on the host).
struct MultTable {
  float v[kMaxPts];
};

// Left shifts applied to the codes of M before the output bracket when M has
// per-point power-of-two scales (entry p = i*n + j; all zero otherwise).  Four bits per
// entry (a shift is at most kMaxMShift = 8), eight entries per word: a kernel keeps the whole
// table in 8 scalar registers and extracts an entry where it is used, instead of holding up
// to 64 registers live across its loops.
struct ShiftTable {
  uint32_t w[kMaxPts / 8];
  void set(int p, int shift) {
    w[p >> 3] = (w[p >> 3] & ~(15u << ((p & 7) * 4))) | ((uint32_t)shift << ((p & 7) * 4));
  }
#if defined(__HIPCC__)
  // Entry P as a wave-uniform value.  The extraction is kept where it is written (volatile):
  // moved out of a loop, the entries would again occupy one scalar register each.
  template <int P>
  __device__ __forceinline__ int at() const {
    uint32_t r;
    asm volatile("s_bfe_u32 %0, %1, %2" : "=s"(r) : "s"(w[P >> 3]), "n"(((P & 7) * 4) | (4 << 16)) : "scc");
    return (int)r;
  }
#endif
};
constexpr int kMaxMShift = 8;

struct Geometry {
  int N, H, W, C, K;
  int m;        // output tile edge
  int TH, TW;   // tiles per image
  int T;        // total tiles
  int frag;     // 1: U and V are in MFMA-fragment order (below), 0: rows [n*n][T or K][C]
  // division of a tile index (< 2^30) by TW and by TW * TH as multiply-high and shift
  uint32_t mul_tw, sh_tw, mul_im, sh_im;
  // division of a work-group index (< 2^30) by the groups per tile of the one-tile-per-group
  // transform kernels: C / 256 (input), K / 256 (output); 1 where that is not a whole number
  uint32_t mul_cg, sh_cg, mul_kg, sh_kg;
  // division of a work-group index by the 64-channel chunks of a row, ceil(C / 64): the groups
  // of the fragment-order transforms are (four rows, one chunk)
  uint32_t mul_ch, sh_ch;
  // input and output transform: work groups per unit (an image or a run of tiles) when every
  // unit's groups are to run on one XCD (0 = work groups in plain order), and the number of
  // groups covered by that order; set per launch (with_image_groups, with_output_groups)
  int img_blocks, img_blocks_end;
};

// Work-group ids go round-robin over the 8 XCDs, each with a private L2 that keeps its lines
// from one kernel to the next.  A line that one XCD wrote and another one read is expensive to
// write again (the other L2's copy has to be found and dropped), and tiles of an image share
// input lines.  The transforms therefore deal their work groups to XCDs in units: launch slot
// b = 8 q + x (XCD x) takes group (q % G) of unit 8 (q / G) + x, G = groups per unit; the slots
// past the last full set of eight units keep their plain order.  A unit is
//   * fragment order: 32 consecutive tiles, the tile block of the contraction + output kernel,
//     which takes tile block j on XCD j % 8: U is read, and written again by the next call, on
//     the XCD that wrote it;
//   * rows, small layers: an eighth of the tiles, which the contraction kernel and the output
//     transform then give to the same XCD (xcd_chunk_tiles), so that U and M stay in one L2;
//   * rows otherwise: one image (shared input lines enter one L2 once).
#if defined(__HIPCC__)
#define WINO_HOST_DEVICE __host__ __device__ __forceinline__
#else
#define WINO_HOST_DEVICE inline
#endif
WINO_HOST_DEVICE unsigned image_on_one_xcd(const Geometry& g, unsigned b) {
  if (g.img_blocks == 0 || b >= (unsigned)g.img_blocks_end) return b;
  const unsigned x = b & 7, q = b >> 3, G = (unsigned)g.img_blocks;
  const unsigned set = q / G, within = q - set * G;
  return (set * 8 + x) * G + within;
}

// Work groups of 256 lanes for `items` lanes' worth of work.
WINO_HOST_DEVICE unsigned blocks_for(long items) { return (unsigned)((items + 255) / 256); }
// A work group's 256 items are the channels of one tile (and offsets inside one
// image fit 32 bits): the kernels then keep the tile arithmetic in scalar registers.
inline bool whole_tiles(int channels, int H, int W) {
  return channels > 0 && channels % 256 == 0 && (long)H * W * channels < (1L << 31);
}
// Work groups of the operand transforms: 256 consecutive items each in row order; in
// fragment order one per (4 rows, 64-channel chunk).
WINO_HOST_DEVICE unsigned weight_blocks(const Geometry& g) {
  return g.frag ? (unsigned)(((long)g.K >> 2) * ((g.C + 63) >> 6)) : blocks_for((long)g.K * g.C);
}
inline unsigned input_blocks(const Geometry& g) {
  return g.frag ? (unsigned)((((long)g.T + 3) >> 2) * ((g.C + 63) >> 6)) : blocks_for((long)g.T * g.C);
}
// Tile rows of a work group of the contraction kernel: 128, or 64 where fewer than two
// 128-row blocks per compute unit would exist (measured: 7 % on a 4x4 x 512-channel layer with
// 256 tiles; no gain from about two blocks per compute unit on).
inline int contract_tile_rows(const Geometry& g) {
  const int n = g.m + 2;
  const long big_tiles = (long)n * n * ((g.T + 127) / 128) * ((g.K + 127) / 128);
  return big_tiles < 2 * 256 ? 64 : 128;
}
// Row order, one kernel per stage: tiles per XCD when input transform, contraction and output
// transform all give the same eighth of the tiles to an XCD, 0 when they do not.  They do when
// the eighths are whole contraction blocks, both transforms run their one-tile-per-group
// kernels (the ones that can be dealt) and U and M together (n*n T (C + K) bytes) fit the eight
// 4 MiB L2s with room to spare: measured on 8x8 images with 256 channels, 26.9 -> 25.8 us per
// layer at N = 256 (19 MB); but 45.9 -> 47.6 us for F(6,3) on the same images (32 MiB), and
// 229 -> 240 us at N = 4096, where nothing stays in an L2 and the output transform loses by
// reading and writing one long run per XCD.  With the contraction alone renumbered (a
// 128-channel layer, whose transforms keep their plain order) a layer lost 10 %.
constexpr long kAlignedXcdBytes = 24L << 20;
inline long xcd_chunk_tiles(const Geometry& g) {
  const int tt = contract_tile_rows(g), n = g.m + 2;
  if (g.frag || g.T <= 0 || g.T % (8L * tt) != 0) return 0;
  if (!whole_tiles(g.C, g.H, g.W) || !whole_tiles(g.K, g.H, g.W)) return 0;
  return (long)n * n * g.T * ((long)g.C + g.K) <= kAlignedXcdBytes ? g.T / 8 : 0;
}
// Groups of tile rows of the contraction kernel: a unit of its block numbering is (point,
// group), and unit u runs on XCD u % 8.  Aligned with the transforms: 8 groups, group j on XCD j.
// Otherwise the smallest split that spreads n*n points over the 8 XCDs evenly.
inline int contract_tile_groups(const Geometry& g, int tile_rows) {
  const int n = g.m + 2, tblocks = (g.T + tile_rows - 1) / tile_rows;
  if (tile_rows == contract_tile_rows(g) && xcd_chunk_tiles(g) > 0) return 8;
  int tgroups = 1;
  while (tgroups < 8 && (n * n * tgroups) % 8 != 0 && tgroups * 2 <= tblocks) tgroups *= 2;
  return tgroups;
}
// Sets the dealing of `per_unit` work groups per unit over `units` units (off when there are
// fewer than eight units or the numbers do not fit).
inline Geometry with_dealt_units(Geometry g, long per_unit, long units) {
  g.img_blocks = 0, g.img_blocks_end = 0;
  const long end = (units / 8) * 8 * per_unit;
  if (per_unit > 0 && per_unit < (1L << 20) && units >= 8 && end < 0x7fffffffL)
    g.img_blocks = (int)per_unit, g.img_blocks_end = (int)end;
  return g;
}
// Geometry for the input transform's launch (whole: the block-uniform row-order kernel, one
// work group per tile and 256 channels).
inline Geometry with_image_groups(const Geometry& g, bool whole) {
  const long nch = (g.C + 63) >> 6;
  if (g.frag) return with_dealt_units(g, 8 * nch, g.T / 32);
  if (!whole) return with_dealt_units(g, 0, 0);
  if (const long chunk = xcd_chunk_tiles(g)) return with_dealt_units(g, chunk * (g.C / 256), 8);
  return with_dealt_units(g, (long)g.TH * g.TW * (g.C / 256), g.N);
}
// Geometry for the launch of the block-uniform output transform (one work group per tile and
// 256 output channels).
inline Geometry with_output_groups(const Geometry& g) {
  return with_dealt_units(g, xcd_chunk_tiles(g) * (g.K / 256), 8);
}

// q = n / d for n < 2^30.  d a power of two: a shift (mul = 0).  Otherwise, with f = floor(log2 d),
// q = (n * mul) >> (32 + f), mul = floor(2^(32 + f) / d) + 1 < 2^32: the excess
// mul d - 2^(32 + f) is at most d < 2^(f + 1), so n times it stays below 2^(32 + f).
inline void fast_div_setup(uint32_t d, uint32_t* mul, uint32_t* sh) {
  uint32_t f = 0;
  while ((2u << f) <= d) ++f;                      // f = floor(log2 d), d >= 1
  *sh = f;
  *mul = (d & (d - 1)) == 0 ? 0u : (uint32_t)((((unsigned long long)1 << (32 + f)) / d) + 1);
}
inline void geometry_set_divisors(Geometry& g) {
  fast_div_setup((uint32_t)(g.TW > 0 ? g.TW : 1), &g.mul_tw, &g.sh_tw);
  fast_div_setup((uint32_t)(g.TW * g.TH > 0 ? g.TW * g.TH : 1), &g.mul_im, &g.sh_im);
  fast_div_setup((uint32_t)(g.C >= 256 && g.C % 256 == 0 ? g.C / 256 : 1), &g.mul_cg, &g.sh_cg);
  fast_div_setup((uint32_t)(g.K >= 256 && g.K % 256 == 0 ? g.K / 256 : 1), &g.mul_kg, &g.sh_kg);
  fast_div_setup((uint32_t)(g.C > 64 ? (g.C + 63) / 64 : 1), &g.mul_ch, &g.sh_ch);
}
#if defined(__HIPCC__)
// n / d with the pair prepared by fast_div_setup for d (n < 2^30).
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t mul, uint32_t sh) {
  return (mul ? __umulhi(n, mul) : n) >> sh;
}
#endif
#if defined(__HIPCC__)
// tile t -> (image b, tile row ty, tile column tx) with t = (b TH + ty) TW + tx, t < 2^30.
__device__ __forceinline__ void tile_coords(const Geometry& g, int t, int& b, int& ty, int& tx) {
  const uint32_t im = (uint32_t)(g.TW * g.TH);
  b = (int)((g.mul_im ? __umulhi((uint32_t)t, g.mul_im) : (uint32_t)t) >> g.sh_im);
  const uint32_t r = (uint32_t)t - (uint32_t)b * im;
  ty = (int)((g.mul_tw ? __umulhi(r, g.mul_tw) : r) >> g.sh_tw);
  tx = (int)(r - (uint32_t)ty * (uint32_t)g.TW);
}
#endif

// Fragment order of a transformed operand X[p][row][c] (rows = tiles for U, output channels
// for V): rows in groups of 16 (RG = ceil(rows / 16) groups), channels in chunks of 64
// (NCH = ceil(C / 64) chunks); the 16 x 64 block of (group, chunk) is one contiguous KiB laid
// out [c % 64 / 16][row % 16][c % 16], which is exactly the register layout of a 16x16x64
// int8 MFMA operand: lane l of a wave reads bytes [16 l, 16 l + 16) of the block.
//   offset(p, row, c) = ((p RG + row / 16) NCH + c / 64) 1024 + (c % 64 / 16) 256 + (row % 16) 16 + c % 16
// Rows past the last one are never written (they only feed results that are discarded);
// channels past C hold zeros in V (and anything in U).
inline long frag_bytes(long n2, long rows, long C) {
  return n2 * ((rows + 15) / 16) * ((C + 63) / 64) * 1024;
}

struct StageMults {
  MultTable inner;   // inner bracket of eq. 2 / eq. 4 (unused when !inner)
  MultTable outer;   // outer bracket, or the only one for the canonical base
};

// Per-M launchers of the transform stages (defined in wino_transforms.hpp and
// instantiated once per M in its own translation unit).
// brackets: 0 = one bracket per stage (canonical matrices); 1, 2, 3 = the two-bracket form of
// eq. 2 / eq. 4 in the monic Legendre, Chebyshev, Hermite base.
template <int M>
struct PerM {
  static hipError_t weight(const Geometry& g, int brackets, const int8_t* w, int8_t* V,
                           const StageMults& mu, hipStream_t st);
  static hipError_t input(const Geometry& g, int brackets, const int8_t* x, int8_t* U,
                          const StageMults& mu, hipStream_t st);
  static hipError_t operands(const Geometry& g, int brackets, const int8_t* x, int8_t* U,
                             const int8_t* w, int8_t* V, const StageMults& mu_in,
                             const StageMults& mu_w, hipStream_t st);
  // sh != nullptr: M carries per-point shifts (8- or 9-bit M only)
  static hipError_t output(const Geometry& g, int brackets, const void* M_, int m_bits,
                           void* y, int out_type, bool relu, const StageMults& mu,
                           const ShiftTable* sh, hipStream_t st);
};
extern template struct PerM<2>;
extern template struct PerM<4>;
extern template struct PerM<6>;

// Calibration launchers (wino_calibrate.hpp): per-(i, j) maxima of the integer
// numerators of one bracket, merged into amax[64] (device, zeroed by the caller).
template <int M>
struct PerMCal {
  static hipError_t weight(const Geometry& g, bool legendre_inner, int phase, const int8_t* w,
                           unsigned long long* amax, const StageMults& mu, hipStream_t st);
  static hipError_t input(const Geometry& g, bool legendre_inner, int phase, const int8_t* x,
                          unsigned long long* amax, const StageMults& mu, hipStream_t st);
  static hipError_t output(const Geometry& g, bool legendre_inner, int phase, const void* M_,
                           int m_bits, unsigned long long* amax, const StageMults& mu, bool relu,
                           const ShiftTable* sh, hipStream_t st);
};
extern template struct PerMCal<2>;
extern template struct PerMCal<4>;
extern template struct PerMCal<6>;

// Run-time fp32 matrices of the trainable brackets (Section 4.2, "flex"),
// row-major with their own column counts: GP n x 3, BPT n x n, APT m x n.
struct FlexMats {
  float GP[8 * 3];
  float BPT[8 * 8];
  float APT[6 * 8];
};

// Launchers of the flex kernels (wino_flex.hpp).  mode 0 runs the stage, 1
// reduces max |fp32 bracket value| into amax[0] (float bit pattern), 2 (weights,
// Legendre) reduces the per-(i, j) numerator maxima of the P^{-1} bracket.
template <int M>
struct PerMFlex {
  static hipError_t weight(const Geometry& g, bool legendre, int mode, const int8_t* w, int8_t* V,
                           unsigned long long* amax, const FlexMats& fm, const StageMults& mu,
                           float mult_first, hipStream_t st);
  static hipError_t input(const Geometry& g, bool legendre, int mode, const int8_t* x, int8_t* U,
                          unsigned long long* amax, const FlexMats& fm, const StageMults& mu,
                          float mult_u, hipStream_t st);
  static hipError_t output(const Geometry& g, bool legendre, int mode, const void* M_, int m_bits,
                           void* y, int out_type, bool relu, unsigned long long* amax,
                           const FlexMats& fm, const StageMults& mu, float mult_out,
                           hipStream_t st);
  // input and weight stage (mode 0) in one launch
  static hipError_t operands(const Geometry& g, bool legendre, const int8_t* x, int8_t* U,
                             const int8_t* w, int8_t* V, const FlexMats& fm,
                             const StageMults& mu_in, float mult_u, const StageMults& mu_w,
                             float mult_first, hipStream_t st);
};
extern template struct PerMFlex<2>;
extern template struct PerMFlex<4>;
extern template struct PerMFlex<6>;

// stage 0 weight, 1 input, 2 output, dispatched on g.m.
hipError_t launch_flex_stage(int stage, const Geometry& g, bool legendre, int mode, const void* in,
                             int m_bits, void* out, int out_type, bool relu,
                             unsigned long long* amax, const FlexMats& fm, const StageMults& mu,
                             float mult, hipStream_t st);

// Input and weight stage of a flex layer in one launch (both outputs non-empty).
hipError_t launch_flex_operands(const Geometry& g, bool legendre, const int8_t* x, int8_t* U,
                                const int8_t* w, int8_t* V, const FlexMats& fm,
                                const StageMults& mu_in, float mult_u, const StageMults& mu_w,
                                float mult_first, hipStream_t st);

// stage: 0 weight, 1 input, 2 output; phase 1 = inner bracket, 2 = outer bracket.
hipError_t launch_calibrate_stage(int stage, const Geometry& g, bool legendre_inner, int phase,
                                  const void* in, int m_bits, unsigned long long* amax,
                                  const StageMults& mu, bool relu, const ShiftTable* sh,
                                  hipStream_t st);
// amax[s] = max |v[s * count + i]|, i < count, for each of `segments` consecutive
// int32 arrays (device pointers).
hipError_t launch_absmax_i32(const int32_t* v, long count, int segments,
                             unsigned long long* amax, hipStream_t st);

// brackets: 0 = the single-bracket form (canonical, or a base with its brackets multiplied
// out); 1 / 2 / 3 = the two-bracket pipeline in the Legendre / Chebyshev / Hermite base.
hipError_t launch_weight_transform(const Geometry& g, int brackets, const int8_t* w,
                                   int8_t* V, const StageMults& mu, hipStream_t st);
hipError_t launch_input_transform(const Geometry& g, int brackets, const int8_t* x,
                                  int8_t* U, const StageMults& mu, hipStream_t st);
// Input and weight transform in one launch (both outputs non-empty).
hipError_t launch_operand_transforms(const Geometry& g, int brackets, const int8_t* x,
                                     int8_t* U, const int8_t* w, int8_t* V,
                                     const StageMults& mu_in, const StageMults& mu_w,
                                     hipStream_t st);
// m_bits: 8 -> int8 M, 9 -> int16 M, 32 -> int32 M (no cast).
// mult.v[p]: multiplier of the cast of point p (unused for m_bits = 32).
hipError_t launch_contract(const Geometry& g, const int8_t* U, const int8_t* V, void* M,
                           int m_bits, const MultTable& mult, hipStream_t st);
// out_type: 0 fp32 (outer table = dequantisation factors), 1 int32 numerators,
// 2 int8 codes (outer table = cast multipliers).
hipError_t launch_output_transform(const Geometry& g, int brackets, const void* M,
                                   int m_bits, void* y, int out_type, bool relu,
                                   const StageMults& mu, const ShiftTable* sh, hipStream_t st);

// Contraction and output transform in one kernel, M kept in LDS (wino_conout.hpp);
// m_bits 8 or 9, out_type 0 or 2, C > 0; U and V in rows or fragment order (g.frag).
template <int M>
struct PerMCO {
  static hipError_t run(const Geometry& g, bool legendre_inner, const int8_t* U, const int8_t* V,
                        void* y, int m_bits, int out_type, bool relu, const StageMults& out_mu,
                        const MultTable& mm, const ShiftTable* sh, hipStream_t st);
  static long blocks(const Geometry& g, int m_bits);
};
// Work groups launch_contract_output would start for this geometry.
long contract_output_blocks(const Geometry& g, int m_bits);
extern template struct PerMCO<2>;
extern template struct PerMCO<4>;
extern template struct PerMCO<6>;
hipError_t launch_contract_output(const Geometry& g, bool legendre_inner, const int8_t* U,
                                  const int8_t* V, void* y, int m_bits, int out_type, bool relu,
                                  const StageMults& out_mu, const MultTable& mm,
                                  const ShiftTable* sh, hipStream_t st);
// Zero fill of `bytes` (a multiple of 16) at a 16-byte aligned device address, by a kernel.
hipError_t launch_fill_zero(void* dst, long bytes, hipStream_t st);

// Fused variant (input transform + contraction + output transform in one kernel);
// V is the transformed filter tensor.  m = 2 or 4, m_bits 8 or 9, out_type 0 or 2.
// mm: cast multiplier of the contraction per point; sh: per-point shifts or null.
hipError_t launch_fused(const Geometry& g, bool legendre_inner, const int8_t* x, const int8_t* V,
                        void* y, int m_bits, int out_type, bool relu, const StageMults& in_mu,
                        const StageMults& out_mu, const MultTable& mm, const ShiftTable* sh,
                        hipStream_t st);

// Backward pass (wino_backward.hip), fp32.  which: 0 dY -> dM, 1 dU -> dx.
hipError_t launch_backward_transform(int which, const Geometry& g, const float* in, float* out,
                                     hipStream_t st);
// Number of partial sums (a power of two, 1 ... 32) the dV contraction leaves for this
// shape; the dV buffer holds that many [n*n][K][C] tensors.  Up to eight are added, into the
// first one, by whichever kernel reads dV next (backward_dv_reader_parts says how many it
// will find); more are added by launch_backward_sum_splits, which launches nothing otherwise.
int backward_dv_splits(const Geometry& g);
int backward_dv_reader_parts(const Geometry& g);
hipError_t launch_backward_sum_splits(const Geometry& g, float* dV, hipStream_t st);
// dV -> dw alone, and dU -> dx with dV -> dw in one launch (both non-empty).
hipError_t launch_backward_dw(const Geometry& g, float* dV, float* dw, hipStream_t st);
hipError_t launch_backward_dx_dw(const Geometry& g, const float* dU, float* dx, float* dV,
                                 float* dw, hipStream_t st);
// for_weights = false: out = dU[p][t][c] = scale[p] sum_k dM[p][t][k] codes[p][k][c] (codes = V);
// for_weights = true:  out = dV[p][k][c] = scale[p] sum_t dM[p][t][k] codes[p][t][c] (codes = U).
hipError_t launch_backward_gemm(bool for_weights, const Geometry& g, const float* dM,
                                const int8_t* codes, float* out, const MultTable& scale,
                                hipStream_t st);

// Backward pass of the flex layer (wino_flex_backward.hpp).  `part` receives one row
// of 64 floats per work group (the group's share of the matrix gradient).
template <int M>
struct PerMFlexBwd {
  static hipError_t output(const Geometry& g, bool legendre, const void* M_, int m_bits,
                           const float* dy, float* dM, float* part, const FlexMats& fm,
                           const StageMults& mu, float s_in, hipStream_t st);
  static hipError_t input_weight(const Geometry& g, bool legendre, const int8_t* x,
                                 const float* dU, float* dXt, float* part_in, const int8_t* w,
                                 float* dV, float* dw, float* part_w, const FlexMats& fm,
                                 const StageMults& mu, float s_in, float s_w, hipStream_t st);
  static hipError_t tile_sum(const Geometry& g, const float* dXt, float* dx, hipStream_t st);
};
extern template struct PerMFlexBwd<2>;
extern template struct PerMFlexBwd<4>;
extern template struct PerMFlexBwd<6>;
// The launches of the flex backward pass besides the contractions, dispatched on g.m.
hipError_t launch_flex_backward_output(const Geometry& g, bool legendre, const void* M_, int m_bits,
                                       const float* dy, float* dM, float* part, const FlexMats& fm,
                                       const StageMults& mu, float s_in, hipStream_t st);
hipError_t launch_flex_backward_input_weight(const Geometry& g, bool legendre, const int8_t* x,
                                             const float* dU, float* dXt, float* part_in,
                                             const int8_t* w, float* dV, float* dw,
                                             float* part_w, const FlexMats& fm,
                                             const StageMults& mu, float s_in, float s_w,
                                             hipStream_t st);
hipError_t launch_flex_backward_tile_sum(const Geometry& g, const float* dXt, float* dx,
                                         hipStream_t st);
// For each of three arrays: out[i][v] = sum over r < rows[i] of part[i][r * 64 + v],
// v < count[i], in a fixed order; one launch.
hipError_t launch_sum_partials(const float* const part[3], const long rows[3], const int count[3],
                               float* const out[3], hipStream_t st);

// Both contraction gradients in one launch (falls back to two when one is empty).
hipError_t launch_backward_gemms(const Geometry& g, const float* dM, const int8_t* U,
                                 const int8_t* V, float* dU, float* dV, const MultTable& s_u,
                                 const MultTable& s_v, hipStream_t st);

// Peak probes: kind 0 = int8 MFMA loop (blocks * 4 waves * iters * 4 MFMAs of
// 32x32x32), kind 1 = 24-bit multiply-add loop (blocks * 256 lanes * iters * 8),
// kind 2 = bf16 MFMA loop (blocks * 4 waves * iters * 4 MFMAs of 32x32x16).
hipError_t launch_probe(int kind, int blocks, int iters, int* sink, hipStream_t st);

// fp32 path: stage 0 weight (a = w), 1 input (a = x), 2 contraction (a = U, b = V),
// 3 output (a = M); no casts, float tensors in the int8 path's layouts.
hipError_t launch_stage_f32(int stage, const Geometry& g, bool legendre, const float* a,
                            const float* b, float* out, bool relu, hipStream_t st);

}  // namespace wino
