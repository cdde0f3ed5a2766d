// C ABI of libwino (see include/wino.h): argument validation, host-side
// multiplier tables, workspace carving and kernel dispatch.
#include "../../include/wino.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "wino_kernels.hpp"
#include "wino_tables.hpp"

using namespace wino;

struct wino_matrices {
  MatrixSet ms;
};

namespace {

thread_local std::string g_err;

}  // namespace

namespace wino {
int report_error(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
}  // namespace wino

namespace {

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

int fail_hip(hipError_t e, const char* what) {
  return fail(WINO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

const RMat* pick(const MatrixSet& ms, int which) {
  switch (which) {
    case WINO_MAT_G: return &ms.G;
    case WINO_MAT_BT: return &ms.BT;
    case WINO_MAT_AT: return &ms.AT;
    case WINO_MAT_PT: return &ms.PT;
    case WINO_MAT_PINVT: return &ms.PinvT;
    case WINO_MAT_GP: return &ms.GP;
    case WINO_MAT_BPT: return &ms.BPT;
    case WINO_MAT_APT: return &ms.APT;
  }
  return nullptr;
}

// Stage matrices of one standard instance, as run-time references.
struct Stages {
  const IMat *G, *BT, *AT, *PinvT, *Pinv, *GP, *BPT, *APT;
};

template <int M, int BASE>
Stages stages_of() {
  using TB = Tab<M, BASE>;
  return Stages{&TB::G, &TB::BT, &TB::AT, &TB::PinvT, &TB::Pinv, &TB::GP, &TB::BPT, &TB::APT};
}

template <int M>
Stages stages_of_base(int base) {
  switch (base) {
    case WINO_BASE_CHEBYSHEV: return stages_of<M, 2>();
    case WINO_BASE_HERMITE: return stages_of<M, 3>();
  }
  return stages_of<M, 1>();     // canonical: G, B^T, A^T are the same in every base
}

bool stages_for(int m, int base, Stages* s) {
  switch (m) {
    case 2: *s = stages_of_base<2>(base); return true;
    case 4: *s = stages_of_base<4>(base); return true;
    case 6: *s = stages_of_base<6>(base); return true;
  }
  return false;
}

// mult_ij = float( s_prev / ( (rho_i rho_j) * s_next ) ), evaluated in double.
// s_next_pt != nullptr: one target scale per entry (per-point scales) instead of s_next.
void fill_mults(MultTable* t, const IMat& im, double s_prev, double s_next,
                const float* s_next_pt = nullptr) {
  std::memset(t, 0, sizeof *t);
  for (int i = 0; i < im.rows; ++i)
    for (int j = 0; j < im.rows; ++j) {
      const double rr = (double)(im.rho[i] * im.rho[j]);
      const double sn = s_next_pt ? (double)s_next_pt[i * im.rows + j] : s_next;
      t->v[i * im.rows + j] = (float)(s_prev / (rr * sn));
    }
}

bool good_scales(const float* s, int count) {
  for (int i = 0; i < count; ++i)
    if (!(std::isfinite(s[i]) && s[i] > 0.f)) return false;
  return true;
}

bool good_scale(float s) { return std::isfinite(s) && s > 0.f; }

// Per-point scales (wino_scales_t.per_point) are an option of the int8 path
// with a cast Hadamard stage and fp32 or int8 output.
int check_per_point(const wino_conv_desc_t* d, const wino_scales_t* s);

struct Plan {
  Geometry g;
  Stages st;
  bool two_brackets;   // a polynomial base with casts on the inner brackets
  int br;              // 0: one bracket per stage; else the base of the two-bracket form (WINO_BASE_*)
  int m_bits;
  bool fp32;           // bits_in = 32: float tensors, no cast anywhere
  bool legendre;
};

int make_plan(const wino_conv_desc_t* d, Plan* p) {
  if (!d) return fail(WINO_EINVAL, "null descriptor");
  if (d->r != 3 || !(d->m == 2 || d->m == 4 || d->m == 6))
    return fail(WINO_EUNSUPPORTED, "F(%d,%d) not built: m must be 2, 4 or 6 and r = 3", d->m, d->r);
  if (d->base < WINO_BASE_CANONICAL || d->base > WINO_BASE_HERMITE)
    return fail(WINO_EINVAL, "unknown base %d", d->base);
  if (d->bits_in != 8 && d->bits_in != 32)
    return fail(WINO_EUNSUPPORTED, "bits_in must be 8 or 32 (got %d)", d->bits_in);
  p->fp32 = d->bits_in == 32;
  if (p->fp32 && d->out_type != WINO_OUT_F32)
    return fail(WINO_EUNSUPPORTED, "the fp32 path (bits_in = 32) has fp32 output only");
  if (!p->fp32 && d->bits_hadamard != 8 && d->bits_hadamard != 9 && d->bits_hadamard != 32)
    return fail(WINO_EUNSUPPORTED, "bits_hadamard must be 8, 9 or 32 (got %d)", d->bits_hadamard);
  if (d->out_type != WINO_OUT_F32 && d->out_type != WINO_OUT_I32 && d->out_type != WINO_OUT_I8)
    return fail(WINO_EINVAL, "unknown out_type %d", d->out_type);
  if (d->N < 0 || d->H < 0 || d->W < 0 || d->C < 0 || d->K < 0)
    return fail(WINO_EINVAL, "negative dimension");
  if (d->C % 16 != 0 || d->K % 16 != 0)
    return fail(WINO_EINVAL, "C (%d) and K (%d) must be multiples of 16", d->C, d->K);
  if (d->C > (1 << 20) || d->K > (1 << 20))   // kernels keep 128 rows of C or K in 32-bit offsets
    return fail(WINO_EINVAL, "C and K must not exceed 2^20");
  const long TH = (d->H + d->m - 1) / d->m, TW = (d->W + d->m - 1) / d->m;
  const long T = (long)d->N * TH * TW;
  const long n2 = (long)(d->m + 2) * (d->m + 2);
  if (T > (1L << 30) || T * (long)(d->C > d->K ? d->C : d->K) * n2 > (1L << 40) ||
      (long)d->N * d->H * d->W * (long)(d->C > d->K ? d->C : d->K) > (1L << 40))
    return fail(WINO_EINVAL, "problem too large");
  if (!p->fp32 && d->bits_hadamard == 32 && d->C > kMaxChannelsExact)
    return fail(WINO_EOVERFLOW, "C = %d: an unquantised contraction result may exceed 2^24", d->C);
  if (d->operand_layout != WINO_LAYOUT_ROWS && d->operand_layout != WINO_LAYOUT_FRAGMENTS)
    return fail(WINO_EINVAL, "unknown operand_layout %d", d->operand_layout);
  if (d->operand_layout == WINO_LAYOUT_FRAGMENTS && p->fp32)
    return fail(WINO_EUNSUPPORTED, "fragment order is a layout of the int8 operands");
  p->g = Geometry{};   // divisors and the XCD dealing are filled in below / by the launchers
  p->g.N = d->N, p->g.H = d->H, p->g.W = d->W, p->g.C = d->C, p->g.K = d->K, p->g.m = d->m;
  p->g.TH = (int)TH, p->g.TW = (int)TW, p->g.T = (int)T;
  p->g.frag = d->operand_layout == WINO_LAYOUT_FRAGMENTS ? 1 : 0;
  geometry_set_divisors(p->g);
  if (!stages_for(d->m, d->base, &p->st)) return fail(WINO_EUNSUPPORTED, "m = %d", d->m);
  p->two_brackets = d->base != WINO_BASE_CANONICAL && d->inner_quant != 0;
  p->br = p->two_brackets ? d->base : 0;
  if (p->fp32 && d->base > WINO_BASE_LEGENDRE)
    return fail(WINO_EUNSUPPORTED, "the fp32 path is built for the canonical and the Legendre base");
  p->m_bits = p->fp32 ? 32 : d->bits_hadamard;
  p->legendre = d->base != WINO_BASE_CANONICAL;
  if (d->out_type == WINO_OUT_I32) {
    const IMat& a = *p->st.AT;
    bool integer = !p->two_brackets;
    for (int i = 0; i < a.rows; ++i) integer = integer && a.rho[i] == 1;
    if (!integer)
      return fail(WINO_EUNSUPPORTED, "int32 output needs an integer output matrix "
                                     "(canonical base or inner_quant = 0, m = 2 or 4)");
  }
  return WINO_OK;
}

int need(const void* p, const char* name) {
  return p ? WINO_OK : fail(WINO_EINVAL, "null pointer: %s", name);
}

// Bytes of V and U in rows or fragment order.
size_t v_bytes_of(const Plan& p, bool frag) {
  const size_t n2 = (size_t)(p.g.m + 2) * (p.g.m + 2);
  return frag ? (size_t)frag_bytes((long)n2, p.g.K, p.g.C) : n2 * p.g.K * p.g.C * (p.fp32 ? 4 : 1);
}
size_t u_bytes_of(const Plan& p, bool frag) {
  const size_t n2 = (size_t)(p.g.m + 2) * (p.g.m + 2);
  return frag ? (size_t)frag_bytes((long)n2, p.g.T, p.g.C) : n2 * p.g.T * p.g.C * (p.fp32 ? 4 : 1);
}

// Fragment order pads the channels of V to a multiple of 64 with zeros (the contraction reads
// whole 64-channel chunks of both operands): when C is not such a multiple the tensor is
// cleared before the transform writes the real channels.
int clear_v_padding(const Plan& p, void* V, void* hip_stream) {
  if (!p.g.frag || p.g.C % 64 == 0 || (long)p.g.K * p.g.C == 0) return WINO_OK;
  hipError_t e = launch_fill_zero(V, (long)v_bytes_of(p, true), (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "zero fill of V");
}

// The Chebyshev and Hermite bases run in the four stage kernels (and the whole-layer call
// built on them); the other variants are built for the canonical and the Legendre base.
int legendre_only(const Plan& p, const char* who) {
  return p.br > WINO_BASE_LEGENDRE
             ? fail(WINO_EUNSUPPORTED, "%s is built for the canonical and the Legendre base", who)
             : WINO_OK;
}

int rows_only(const Plan& p, const char* who) {
  return p.g.frag ? fail(WINO_EUNSUPPORTED, "%s takes U and V in WINO_LAYOUT_ROWS only", who)
                  : WINO_OK;
}

int aligned(const void* p, size_t a, const char* name) {
  return ((uintptr_t)p % a) == 0 ? WINO_OK
                                 : fail(WINO_EINVAL, "%s must be %zu-byte aligned", name, a);
}

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t m_elem_bytes(int bits) { return bits == 8 ? 1 : bits == 9 ? 2 : 4; }

int check_per_point(const wino_conv_desc_t* d, const wino_scales_t* s) {
  if (!s || !s->per_point) return WINO_OK;
  if (s->per_point != 1) return fail(WINO_EINVAL, "per_point must be 0 or 1");
  if (d->bits_in != 8 || (d->bits_hadamard != 8 && d->bits_hadamard != 9))
    return fail(WINO_EUNSUPPORTED, "per-point scales need the int8 path with bits_hadamard 8 or 9");
  if (d->out_type == WINO_OUT_I32)
    return fail(WINO_EUNSUPPORTED, "per-point scales have fp32 or int8 output");
  return WINO_OK;
}

int weight_mults(const Plan& p, const wino_scales_t* s, StageMults* mu) {
  const int n2 = (p.g.m + 2) * (p.g.m + 2);
  const bool pp = s->per_point != 0;
  if (!good_scale(s->s_w) || !(pp ? good_scales(s->s_v_pt, n2) : good_scale(s->s_v)))
    return fail(WINO_EINVAL, "bad s_w / s_v");
  const float* vpt = pp ? s->s_v_pt : nullptr;
  if (p.two_brackets) {
    if (!good_scale(s->s_w1)) return fail(WINO_EINVAL, "bad s_w1");
    fill_mults(&mu->inner, *p.st.GP, s->s_w, s->s_w1);
    fill_mults(&mu->outer, *p.st.Pinv, s->s_w1, s->s_v, vpt);
  } else {
    fill_mults(&mu->outer, *p.st.G, s->s_w, s->s_v, vpt);
  }
  return WINO_OK;
}

int input_mults(const Plan& p, const wino_scales_t* s, StageMults* mu) {
  const int n2 = (p.g.m + 2) * (p.g.m + 2);
  const bool pp = s->per_point != 0;
  if (!good_scale(s->s_x) || !(pp ? good_scales(s->s_u_pt, n2) : good_scale(s->s_u)))
    return fail(WINO_EINVAL, "bad s_x / s_u");
  const float* upt = pp ? s->s_u_pt : nullptr;
  if (p.two_brackets) {
    if (!good_scale(s->s_x1)) return fail(WINO_EINVAL, "bad s_x1");
    fill_mults(&mu->inner, *p.st.PinvT, s->s_x, s->s_x1);
    fill_mults(&mu->outer, *p.st.BPT, s->s_x1, s->s_u, upt);
  } else {
    fill_mults(&mu->outer, *p.st.BT, s->s_x, s->s_u, upt);
  }
  return WINO_OK;
}

// Cast multipliers of the contraction, one per point, the left shifts that
// bring the codes of M to one scale (per-point mode; null = not wanted) and
// that scale: what one unit fed to the output bracket stands for.
int contract_mults(const Plan& p, const wino_scales_t* s, MultTable* mult, ShiftTable* sh,
                   double* s_fed) {
  const int n2 = (p.g.m + 2) * (p.g.m + 2);
  std::memset(mult, 0, sizeof *mult);
  if (sh) std::memset(sh, 0, sizeof *sh);
  if (!s->per_point) {
    if (!good_scale(s->s_u) || !good_scale(s->s_v)) return fail(WINO_EINVAL, "bad s_u / s_v");
    const double s_uv = (double)s->s_u * (double)s->s_v;
    float m = 1.f;
    *s_fed = s_uv;
    if (p.m_bits != 32) {
      if (!good_scale(s->s_m)) return fail(WINO_EINVAL, "bad s_m");
      m = (float)(s_uv / (double)s->s_m);
      *s_fed = (double)s->s_m;
    }
    for (int q = 0; q < n2; ++q) mult->v[q] = m;
    return WINO_OK;
  }
  if (!good_scales(s->s_u_pt, n2) || !good_scales(s->s_v_pt, n2) || !good_scale(s->s_m))
    return fail(WINO_EINVAL, "bad per-point s_u / s_v or s_m");
  int smax = 0;
  for (int q = 0; q < n2; ++q) {
    if (s->m_shift[q] < 0 || s->m_shift[q] > kMaxMShift)
      return fail(WINO_EINVAL, "m_shift[%d] = %d outside 0..%d", q, s->m_shift[q], kMaxMShift);
    if (s->m_shift[q] > smax) smax = s->m_shift[q];
  }
  for (int q = 0; q < n2; ++q) {
    const double s_uv = (double)s->s_u_pt[q] * (double)s->s_v_pt[q];
    mult->v[q] = (float)(s_uv * std::ldexp(1.0, s->m_shift[q]) / (double)s->s_m);
    if (sh) sh->set(q, smax - s->m_shift[q]);
  }
  *s_fed = std::ldexp((double)s->s_m, -smax);
  return WINO_OK;
}

int output_mults(const Plan& p, const wino_conv_desc_t* d, const wino_scales_t* s,
                 StageMults* mu, ShiftTable* sh) {
  MultTable dummy;
  double s_m;
  if (int rc = contract_mults(p, s, &dummy, sh, &s_m)) return rc;
  double s_next = 1.0;   // fp32 output: the table holds dequantisation factors
  if (d->out_type == WINO_OUT_I8) {
    if (!good_scale(s->s_y)) return fail(WINO_EINVAL, "bad s_y");
    s_next = (double)s->s_y;
  }
  if (p.two_brackets) {
    if (!good_scale(s->s_m1)) return fail(WINO_EINVAL, "bad s_m1");
    fill_mults(&mu->inner, *p.st.PinvT, s_m, s->s_m1);
    fill_mults(&mu->outer, *p.st.APT, s->s_m1, s_next);
  } else {
    fill_mults(&mu->outer, *p.st.AT, s_m, s_next);
  }
  return WINO_OK;
}

// Which kernels wino_conv2d runs for a descriptor.
enum Path {
  kPathSplit,      // one kernel per stage: (operand transforms,) contraction, output transform
  kPathFusedAll,   // input transform + contraction + output transform in one kernel
  kPathConOut      // input transform, then contraction + output transform in one kernel
};

// Tuning option (wino_set_option), process-wide.
int g_opt_auto_conout = 1;   // AUTO may take the contraction + output kernel

// The variants that keep M on chip cover the int8 path with a cast Hadamard stage and fp32 or
// int8 output; the single-kernel variant additionally needs m = 2 or 4.  C = 0 (an empty
// channel sum, y = 0) always runs stage by stage.
bool conout_covers(const wino_conv_desc_t* d, const Plan& p) {
  return !(p.fp32 || p.m_bits == 32 || d->out_type == WINO_OUT_I32 || d->C == 0 ||
           p.br > WINO_BASE_LEGENDRE);
}
bool fused_all_covers(const wino_conv_desc_t* d, const Plan& p) {
  return conout_covers(d, p) && d->m != 6;
}

// AUTO takes the two-kernel form where it was measured to be the faster one.  It saves the M
// round trip and a launch; it pays with operands re-read through the L2 four times as often
// (32 x 32 blocks against the 128 x 128 tiles of the stand-alone contraction) and with
// operand transforms that are about 5 % slower into fragment order.  Its tile blocks run on the
// XCD whose input-transform work groups wrote their U (image_on_one_xcd), which is what makes it
// the faster form on layers that fit the L2s.  Measured, whole layer, fp32 y, two-kernel form
// against one kernel per stage (us):
//  * C <= 128: it wins at every size tried, with raw or transformed filters, fp32 or int8
//    output: 16x16 images, C = K = 128, N = 32 / 256 / 2048: 16.5 / 30.7 / 216 against
//    17.6 / 37.0 / 227; C = 64, K = 128: 26 against 31; C = 128, K = 256: 52 against 54.
//    (A block's operand bytes go with C, its output brackets do not, and the stand-alone
//    kernels waste half of their 128-byte channel chunks and 128-wide k blocks on such
//    layers.)
//  * 128 < C <= 256, 8-bit M: it wins where the grid is about one work group per compute unit
//    (8x8 images, C = K = 256, raw filters, N = 192 / 256: 22.0 / 24.2 against 23.2 / 25.6 --
//    23.0 against 24.6 at N = 256 since the filter work groups lead the operand launch;
//    filters transformed: 18.4 / 21.4 against 21.9 / 22.4), and loses on smaller and on larger
//    grids (N = 64 / 128 / 320 / 512 / 1024 / 4096, raw filters: 19.9 / 21.0 / 32.8 / 42.6 / 75.8 /
//    263 against 17.0 / 19.9 / 28.4 / 39.7 / 68.4 / 229).
//  * 128 < C <= 256, 9-bit M (twice the bytes of M): it wins from 256 to 16384 tiles (N = 256 /
//    1024 / 4096: 24.1 / 74.5 / 263 against 27.6 / 77.5 / 269; N = 16384: 1108 against 1077).
//  * C > 256: a block's operand bytes go with C and it loses (C = K = 512, 4x4 images: 35 against
//    25 at N = 256, 8-bit; C = K = 384, 8x8 images: 47 against 42).
//  * F(6,3): 59 against 48 (its output bracket needs 64-bit arithmetic and runs better at the
//    stand-alone kernel's occupancy).
constexpr int kConOutNarrowC = 128;            // up to here: whenever the grid has kConOutMinBlocksNarrow
constexpr long kConOutMinBlocksNarrow = 64;
constexpr int kConOutWideC = 256;              // up to here: between these block counts, with a 9-bit M,
constexpr long kConOutMinBlocks = 192;         // or with an 8-bit M when the grid is about one work
constexpr long kConOutMaxBlocks8 = 256;        // group per compute unit
constexpr long kConOutMaxBlocks9 = 4096;

bool auto_takes_conout(const wino_conv_desc_t* d, const Plan& p) {
  const long blocks = contract_output_blocks(p.g, p.m_bits);
  if (d->C <= kConOutNarrowC) return blocks >= kConOutMinBlocksNarrow;
  if (d->C > kConOutWideC || blocks < kConOutMinBlocks) return false;
  return blocks <= (p.m_bits == 9 ? kConOutMaxBlocks9 : kConOutMaxBlocks8);
}

// ON: M never leaves the chip.  The single kernel where the layer has one 64-channel chunk
// (its input transform is recomputed per 64 output channels and it keeps no accumulators
// across chunks), the two-kernel form otherwise.  AUTO: whichever form is the fastest for the
// shape: the single kernel for C, K <= 64, the two-kernel form for every other covered layer
// that is large enough.
int select_path(const wino_conv_desc_t* d, const Plan& p, Path* path) {
  *path = kPathSplit;
  if (d->fused != WINO_FUSED_OFF && d->fused != WINO_FUSED_ON && d->fused != WINO_FUSED_AUTO)
    return fail(WINO_EINVAL, "unknown fused mode %d", d->fused);
  if (d->fused == WINO_FUSED_OFF || d->C == 0) return WINO_OK;
  if (d->fused == WINO_FUSED_ON) {
    if (!conout_covers(d, p))
      return fail(WINO_EUNSUPPORTED, "the fused variants cover the int8 path with bits_hadamard "
                                     "8 or 9 and fp32 or int8 output, in the canonical and the "
                                     "Legendre base");
    *path = (fused_all_covers(d, p) && d->C <= 64 && !p.g.frag) ? kPathFusedAll : kPathConOut;
    return WINO_OK;
  }
  const bool v_rows_given = d->weights_pretransformed && !p.g.frag;   // slow in the two-kernel form
  if (fused_all_covers(d, p) && d->C <= 64 && d->K <= 64 && !p.g.frag)
    *path = kPathFusedAll;
  else if (conout_covers(d, p) && d->weights_pretransformed && p.g.frag)
    *path = kPathConOut;                       // the only form that reads a V in fragment order
  else if (conout_covers(d, p) && g_opt_auto_conout && !v_rows_given && d->m != 6 &&
           auto_takes_conout(d, p))
    *path = kPathConOut;
  return WINO_OK;
}

// Order of U and V inside wino_conv2d: fragments for the two-kernel form unless the caller
// hands over a V in rows; rows everywhere else.  A V in fragment order is only meaningful to
// the two-kernel form.
int conv_layout(const wino_conv_desc_t* d, const Plan& p, Path path, bool* frag) {
  *frag = path == kPathConOut && (!d->weights_pretransformed || p.g.frag);
  if (d->weights_pretransformed && p.g.frag && path != kPathConOut)
    return fail(WINO_EUNSUPPORTED, "a V in fragment order is read by the two-kernel form only "
                                   "(fused = ON or AUTO on a layer it covers)");
  return WINO_OK;
}

}  // namespace

extern "C" {

const char* wino_last_error(void) { return g_err.c_str(); }

int wino_set_option(int option, int value) {
  switch (option) {
    case WINO_OPT_AUTO_CONOUT:
      g_opt_auto_conout = value != 0;
      return WINO_OK;
  }
  return fail(WINO_EINVAL, "unknown option %d", option);
}

int wino_conv2d_launches(const wino_conv_desc_t* d, char* buf, size_t buf_bytes) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (!buf || buf_bytes == 0) return fail(WINO_EINVAL, "null buffer");
  Path path;
  if (int rc = select_path(d, p, &path)) return rc;
  std::string names;
  auto add = [&](const char* nm) { names += names.empty() ? "" : ","; names += nm; };
  if (p.g.T != 0 && p.g.K != 0) {
    const bool w = !d->weights_pretransformed && (long)p.g.K * p.g.C != 0;
    const bool x = (long)p.g.T * p.g.C != 0;
    if (path == kPathFusedAll) {
      if (w) add("weight_transform");
      add("fused_layer");
    } else {
      if (p.fp32) {
        if (w) add("weight_transform");
        if (x) add("input_transform");
      } else if (w && x) {
        add("operand_transforms");
      } else if (w) {
        add("weight_transform");
      } else if (x) {
        add("input_transform");
      }
      if (path == kPathConOut) {
        add("contraction_output");
      } else {
        add("contraction");
        add("output_transform");
      }
    }
  }
  if (names.size() + 1 > buf_bytes) return fail(WINO_EINVAL, "buffer too small");
  std::memcpy(buf, names.c_str(), names.size() + 1);
  return WINO_OK;
}

int wino_backward_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (p.fp32) return fail(WINO_EUNSUPPORTED, "the backward pass takes the int8 path's U and V");
  if (int rc = rows_only(p, "the backward pass")) return rc;
  if (!bytes) return fail(WINO_EINVAL, "null bytes");
  const size_t n2 = (size_t)(d->m + 2) * (d->m + 2);
  const size_t T = (size_t)p.g.T, C = (size_t)d->C, K = (size_t)d->K;
  const size_t splits = (size_t)backward_dv_splits(p.g);
  size_t total = round256(n2 * T * K * 4) + round256(n2 * T * C * 4) + round256(splits * n2 * K * C * 4);
  if (total == 0) total = 256;
  *bytes = total;
  return WINO_OK;
}

int wino_backward_dv_parts(const wino_conv_desc_t* d, int* parts) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (!parts) return fail(WINO_EINVAL, "null parts");
  *parts = backward_dv_splits(p.g);
  return WINO_OK;
}

int wino_backward(const wino_conv_desc_t* d, const void* dy, const void* U, const void* V,
                  const wino_scales_t* s, void* dx, void* dw, void* workspace, size_t ws_bytes,
                  void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  size_t want = 0;
  if (int rc = wino_backward_workspace_bytes(d, &want)) return rc;
  if (int rc = need(s, "scales")) return rc;
  const int n2 = (d->m + 2) * (d->m + 2);
  MultTable su, sv;
  std::memset(&su, 0, sizeof su);
  std::memset(&sv, 0, sizeof sv);
  if (s->per_point) {
    if (s->per_point != 1) return fail(WINO_EINVAL, "per_point must be 0 or 1");
    if (!good_scales(s->s_u_pt, n2) || !good_scales(s->s_v_pt, n2))
      return fail(WINO_EINVAL, "bad per-point s_u / s_v");
    for (int q = 0; q < n2; ++q) su.v[q] = s->s_u_pt[q], sv.v[q] = s->s_v_pt[q];
  } else {
    if (!good_scale(s->s_u) || !good_scale(s->s_v)) return fail(WINO_EINVAL, "bad s_u / s_v");
    for (int q = 0; q < n2; ++q) su.v[q] = s->s_u, sv.v[q] = s->s_v;
  }
  const Geometry& g = p.g;
  const long x_items = (long)g.N * g.H * g.W * g.C, w_items = (long)g.K * g.C;
  if (x_items == 0 && w_items == 0) return WINO_OK;   // nothing to write
  if (int rc = need(workspace, "workspace")) return rc;
  if (ws_bytes < want) return fail(WINO_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, want);
  if ((uintptr_t)workspace % 256) return fail(WINO_EWORKSPACE, "workspace must be 256-byte aligned");
  if (x_items) if (int rc = need(dx, "dx")) return rc;
  if (w_items) if (int rc = need(dw, "dw")) return rc;
  const long y_items = (long)g.N * g.H * g.W * g.K;
  if (y_items) if (int rc = need(dy, "dy")) return rc;
  if ((long)g.T * g.C) if (int rc = need(U, "U")) return rc;
  if (w_items) if (int rc = need(V, "V")) return rc;
  if (int rc = aligned(dy, 16, "dy")) return rc;
  if (int rc = aligned(U, 16, "U")) return rc;
  if (int rc = aligned(V, 16, "V")) return rc;
  const size_t T = (size_t)g.T, C = (size_t)g.C, K = (size_t)g.K;
  char* ws = static_cast<char*>(workspace);
  float* dM = reinterpret_cast<float*>(ws);  ws += round256((size_t)n2 * T * K * 4);
  float* dU = reinterpret_cast<float*>(ws);  ws += round256((size_t)n2 * T * C * 4);
  float* dV = reinterpret_cast<float*>(ws);
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e = launch_backward_transform(0, g, (const float*)dy, dM, st);
  if (e != hipSuccess) return fail_hip(e, "backward dM launch");
  // An empty reduction (K = 0 resp. T = 0) makes the contraction kernels store zeros.
  if ((long)g.T * g.C && w_items && g.K) {
    e = launch_backward_gemms(g, dM, (const int8_t*)U, (const int8_t*)V, dU, dV, su, sv, st);
    if (e != hipSuccess) return fail_hip(e, "backward contraction launch");
  } else {
    if ((long)g.T * g.C) {
      e = launch_backward_gemm(false, g, dM, (const int8_t*)V, dU, sv, st);
      if (e != hipSuccess) return fail_hip(e, "backward dU launch");
    }
    if (w_items) {
      e = launch_backward_gemm(true, g, dM, (const int8_t*)U, dV, su, st);
      if (e != hipSuccess) return fail_hip(e, "backward dV launch");
    }
  }
  if (w_items) {
    e = launch_backward_sum_splits(g, dV, st);          // no launch unless dV came in several parts
    if (e != hipSuccess) return fail_hip(e, "backward partial-sum launch");
  }
  if (w_items && x_items) {
    e = launch_backward_dx_dw(g, dU, (float*)dx, dV, (float*)dw, st);
    if (e != hipSuccess) return fail_hip(e, "backward dx / dw launch");
  } else if (w_items) {
    e = launch_backward_dw(g, dV, (float*)dw, st);
    if (e != hipSuccess) return fail_hip(e, "backward dw launch");
  } else if (x_items) {
    e = launch_backward_transform(1, g, dU, (float*)dx, st);
    if (e != hipSuccess) return fail_hip(e, "backward dx launch");
  }
  return WINO_OK;
}

int wino_profile_next_launch(void* start_event, void* stop_event) {
  set_profile_events((hipEvent_t)start_event, (hipEvent_t)stop_event);
  return WINO_OK;
}

int wino_probe_peak(int kind, int blocks, int iters, void* sink, double* work, void* hip_stream) {
  if (kind != WINO_PROBE_MFMA_I8 && kind != WINO_PROBE_VALU_MAD24 && kind != WINO_PROBE_MFMA_BF16)
    return fail(WINO_EINVAL, "unknown probe %d", kind);
  if (blocks < 1 || blocks > (1 << 20) || iters < 1 || iters > (1 << 24))
    return fail(WINO_EINVAL, "probe size out of range");
  if (int rc = need(sink, "sink")) return rc;
  if (work)
    *work = kind == WINO_PROBE_MFMA_I8    ? (double)blocks * 4.0 * iters * 4.0 * (2.0 * 32 * 32 * 32)
            : kind == WINO_PROBE_MFMA_BF16 ? (double)blocks * 4.0 * iters * 4.0 * (2.0 * 32 * 32 * 16)
                                          : (double)blocks * 256.0 * iters * 8.0;
  hipError_t e = launch_probe(kind, blocks, iters, (int*)sink, (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "probe launch");
}

int wino_make_matrices(int m, int r, const wino_rat_t* points, int n_finite, int base,
                       wino_matrices_t** out) {
  if (!out) return fail(WINO_EINVAL, "null out");
  *out = nullptr;
  if (m < 1 || r < 1) return fail(WINO_EINVAL, "m and r must be positive");
  if (m + r - 1 > kMaxN) return fail(WINO_EUNSUPPORTED, "m + r - 1 = %d exceeds %d", m + r - 1, kMaxN);
  if (n_finite != m + r - 2) return fail(WINO_EINVAL, "need m + r - 2 = %d finite points, got %d", m + r - 2, n_finite);
  if (n_finite > 0 && !points) return fail(WINO_EINVAL, "null points");
  if (base < WINO_BASE_CANONICAL || base > WINO_BASE_HERMITE)
    return fail(WINO_EINVAL, "unknown base %d", base);
  Rat pts[kMaxN];
  for (int i = 0; i < n_finite; ++i) {
    if (points[i].den == 0) return fail(WINO_EINVAL, "point %d has a zero denominator", i);
    pts[i] = make_rat(points[i].num, points[i].den);
    if (!pts[i].ok) return fail(WINO_EOVERFLOW, "point %d out of range", i);
    for (int j = 0; j < i; ++j)
      if (rat_eq(pts[i], pts[j])) return fail(WINO_EINVAL, "points %d and %d coincide", j, i);
  }
  wino_matrices* h = new (std::nothrow) wino_matrices;
  if (!h) return fail(WINO_EINVAL, "out of host memory");
  h->ms = make_matrix_set(m, r, pts, n_finite, base);
  if (!h->ms.ok) {
    delete h;
    return fail(WINO_EOVERFLOW, "a rational overflowed int64 while building F(%d,%d)", m, r);
  }
  *out = h;
  return WINO_OK;
}

void wino_free_matrices(wino_matrices_t* h) { delete h; }

int wino_get_matrix(const wino_matrices_t* h, int which, wino_rat_t* buf, int* rows, int* cols) {
  if (!h || !buf || !rows || !cols) return fail(WINO_EINVAL, "null argument");
  const RMat* mtx = pick(h->ms, which);
  if (!mtx) return fail(WINO_EINVAL, "unknown matrix id %d", which);
  *rows = mtx->rows;
  *cols = mtx->cols;
  for (int i = 0; i < mtx->rows; ++i)
    for (int j = 0; j < mtx->cols; ++j)
      buf[i * mtx->cols + j] = wino_rat_t{mtx->a[i][j].num, mtx->a[i][j].den};
  return WINO_OK;
}

int wino_get_int_form(const wino_matrices_t* h, int which, int64_t* N, int64_t* row_lcd,
                      int* rows, int* cols) {
  if (!h || !N || !row_lcd || !rows || !cols) return fail(WINO_EINVAL, "null argument");
  const RMat* mtx = pick(h->ms, which);
  if (!mtx) return fail(WINO_EINVAL, "unknown matrix id %d", which);
  const IMat im = int_form(*mtx);
  if (!im.ok) return fail(WINO_EOVERFLOW, "integer form overflowed int64");
  *rows = im.rows;
  *cols = im.cols;
  for (int i = 0; i < im.rows; ++i) {
    row_lcd[i] = im.rho[i];
    for (int j = 0; j < im.cols; ++j) N[i * im.cols + j] = im.N[i][j];
  }
  return WINO_OK;
}

int wino_operand_bytes(const wino_conv_desc_t* d, size_t* v_bytes, size_t* u_bytes) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (v_bytes) *v_bytes = v_bytes_of(p, p.g.frag != 0);
  if (u_bytes) *u_bytes = u_bytes_of(p, p.g.frag != 0);
  return WINO_OK;
}

int wino_preferred_operand_layout(const wino_conv_desc_t* d, int* layout) {
  if (!d || !layout) return fail(WINO_EINVAL, "null argument");
  wino_conv_desc_t dd = *d;
  dd.weights_pretransformed = 1;
  dd.fused = WINO_FUSED_AUTO;
  *layout = WINO_LAYOUT_ROWS;
  dd.operand_layout = WINO_LAYOUT_ROWS;
  Plan p;
  if (int rc = make_plan(&dd, &p)) return rc;
  Path path;
  if (int rc = select_path(&dd, p, &path)) return rc;
  if (path == kPathFusedAll || p.fp32) return WINO_OK;   // the single kernel reads V in rows
  // would AUTO take the two-kernel form, on its merits, for filters that arrive transformed?
  if (conout_covers(&dd, p) && g_opt_auto_conout && dd.m != 6 && auto_takes_conout(&dd, p))
    *layout = WINO_LAYOUT_FRAGMENTS;
  return WINO_OK;
}

int wino_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (!bytes) return fail(WINO_EINVAL, "null bytes");
  const size_t n2 = (size_t)(d->m + 2) * (d->m + 2);
  const size_t eb = p.fp32 ? 4 : 1;
  Path path;
  if (int rc = select_path(d, p, &path)) return rc;
  bool frag;
  if (int rc = conv_layout(d, p, path, &frag)) return rc;
  size_t total = 0;
  (void)eb;
  if (!d->weights_pretransformed) total += round256(v_bytes_of(p, frag));
  // U unless the single kernel runs, M only when one kernel runs per stage
  if (path != kPathFusedAll) total += round256(u_bytes_of(p, frag));
  if (path == kPathSplit) total += round256(n2 * p.g.T * d->K * m_elem_bytes(p.m_bits));
  if (total == 0) total = 256;
  *bytes = total;
  return WINO_OK;
}

int wino_weight_transform(const wino_conv_desc_t* d, const void* w, void* V,
                          const wino_scales_t* s, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if ((long)p.g.K * p.g.C == 0) return WINO_OK;   // empty problem: nothing to launch, pointers may be null
  if (int rc = need(w, "w")) return rc;
  if (int rc = need(V, "V")) return rc;
  if (p.fp32) {
    hipError_t e = launch_stage_f32(0, p.g, p.legendre, (const float*)w, (const float*)nullptr,
                                    (float*)V, false, (hipStream_t)hip_stream);
    return e == hipSuccess ? WINO_OK : fail_hip(e, "fp32 weight launch");
  }
  if (int rc = need(s, "scales")) return rc;
  if (int rc = aligned(w, 16, "w")) return rc;
  if (int rc = aligned(V, 16, "V")) return rc;
  if (int rc = check_per_point(d, s)) return rc;
  StageMults mu;
  if (int rc = weight_mults(p, s, &mu)) return rc;
  if (int rc = clear_v_padding(p, V, hip_stream)) return rc;
  hipError_t e = launch_weight_transform(p.g, p.br, (const int8_t*)w, (int8_t*)V, mu,
                                         (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "weight transform launch");
}

int wino_input_transform(const wino_conv_desc_t* d, const void* x, void* U,
                         const wino_scales_t* s, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if ((long)p.g.T * p.g.C == 0) return WINO_OK;   // empty problem: nothing to launch, pointers may be null
  if (int rc = need(x, "x")) return rc;
  if (int rc = need(U, "U")) return rc;
  if (p.fp32) {
    hipError_t e = launch_stage_f32(1, p.g, p.legendre, (const float*)x, (const float*)nullptr,
                                    (float*)U, false, (hipStream_t)hip_stream);
    return e == hipSuccess ? WINO_OK : fail_hip(e, "fp32 input launch");
  }
  if (int rc = need(s, "scales")) return rc;
  if (int rc = aligned(x, 16, "x")) return rc;
  if (int rc = aligned(U, 16, "U")) return rc;
  if (int rc = check_per_point(d, s)) return rc;
  StageMults mu;
  if (int rc = input_mults(p, s, &mu)) return rc;
  hipError_t e = launch_input_transform(p.g, p.br, (const int8_t*)x, (int8_t*)U, mu,
                                        (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "input transform launch");
}

int wino_transform_operands(const wino_conv_desc_t* d, const void* x, void* U, const void* w,
                            void* V, const wino_scales_t* s, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if ((long)p.g.T * p.g.C == 0 && (long)p.g.K * p.g.C == 0) return WINO_OK;   // empty problem: nothing to launch, pointers may be null
  if (p.fp32) {   // the unquantised path keeps its two separate launches
    if (int rc = wino_weight_transform(d, w, V, s, hip_stream)) return rc;
    return wino_input_transform(d, x, U, s, hip_stream);
  }
  if (int rc = need(x, "x")) return rc;
  if (int rc = need(U, "U")) return rc;
  if (int rc = need(w, "w")) return rc;
  if (int rc = need(V, "V")) return rc;
  if (int rc = need(s, "scales")) return rc;
  if (int rc = aligned(x, 16, "x")) return rc;
  if (int rc = aligned(U, 16, "U")) return rc;
  if (int rc = aligned(w, 16, "w")) return rc;
  if (int rc = aligned(V, 16, "V")) return rc;
  if (int rc = check_per_point(d, s)) return rc;
  StageMults mu_in, mu_w;
  if (int rc = input_mults(p, s, &mu_in)) return rc;
  if (int rc = weight_mults(p, s, &mu_w)) return rc;
  if (int rc = clear_v_padding(p, V, hip_stream)) return rc;
  hipError_t e = launch_operand_transforms(p.g, p.br, (const int8_t*)x, (int8_t*)U,
                                           (const int8_t*)w, (int8_t*)V, mu_in, mu_w,
                                           (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "operand transforms launch");
}

int wino_contract(const wino_conv_desc_t* d, const void* U, const void* V, void* M,
                  const wino_scales_t* s, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if ((long)p.g.T * p.g.K == 0) return WINO_OK;   // empty problem: nothing to launch, pointers may be null
  if (p.g.C != 0) {                               // C = 0: U and V are empty and are not read
    if (int rc = need(U, "U")) return rc;
    if (int rc = need(V, "V")) return rc;
  }
  if (int rc = need(M, "M")) return rc;
  if (p.fp32) {
    hipError_t e = launch_stage_f32(2, p.g, p.legendre, (const float*)U, (const float*)V,
                                    (float*)M, false, (hipStream_t)hip_stream);
    return e == hipSuccess ? WINO_OK : fail_hip(e, "fp32 contract launch");
  }
  if (int rc = need(s, "scales")) return rc;
  if (int rc = aligned(U, 16, "U")) return rc;
  if (int rc = aligned(V, 16, "V")) return rc;
  if (int rc = aligned(M, 16, "M")) return rc;
  if (int rc = check_per_point(d, s)) return rc;
  if (int rc = rows_only(p, "wino_contract")) return rc;
  MultTable mult;
  double s_m;
  if (int rc = contract_mults(p, s, &mult, nullptr, &s_m)) return rc;
  hipError_t e = launch_contract(p.g, (const int8_t*)U, (const int8_t*)V, M, p.m_bits, mult,
                                 (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "contraction launch");
}

int wino_output_transform(const wino_conv_desc_t* d, const void* M, void* y,
                          const wino_scales_t* s, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if ((long)p.g.T * p.g.K == 0) return WINO_OK;   // empty problem: nothing to launch, pointers may be null
  if (int rc = need(M, "M")) return rc;
  if (int rc = need(y, "y")) return rc;
  if (p.fp32) {
    hipError_t e = launch_stage_f32(3, p.g, p.legendre, (const float*)M, (const float*)nullptr,
                                    (float*)y, d->relu != 0, (hipStream_t)hip_stream);
    return e == hipSuccess ? WINO_OK : fail_hip(e, "fp32 output launch");
  }
  if (int rc = need(s, "scales")) return rc;
  if (int rc = aligned(M, 16, "M")) return rc;
  if (int rc = aligned(y, 16, "y")) return rc;
  if (int rc = check_per_point(d, s)) return rc;
  if (p.br > WINO_BASE_LEGENDRE && s->per_point)
    return fail(WINO_EUNSUPPORTED, "per-point scales are built for the canonical and the Legendre base");
  StageMults mu;
  ShiftTable sh;
  if (int rc = output_mults(p, d, s, &mu, &sh)) return rc;
  hipError_t e = launch_output_transform(p.g, p.br, M, p.m_bits, y, d->out_type,
                                         d->relu != 0, mu, s->per_point ? &sh : nullptr,
                                         (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "output transform launch");
}

int wino_contract_output(const wino_conv_desc_t* d, const void* U, const void* V, void* y,
                         const wino_scales_t* s, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if ((long)p.g.T * p.g.K == 0) return WINO_OK;   // no output element exists
  if (p.fp32 || p.m_bits == 32 || d->out_type == WINO_OUT_I32)
    return fail(WINO_EUNSUPPORTED, "contraction + output transform in one kernel covers the int8 "
                                   "path with bits_hadamard 8 or 9 and fp32 or int8 output");
  if (int rc = legendre_only(p, "wino_contract_output")) return rc;
  if (p.g.C != 0) {                               // C = 0: U and V are empty and are not read
    if (int rc = need(U, "U")) return rc;
    if (int rc = need(V, "V")) return rc;
  }
  if (int rc = need(y, "y")) return rc;
  if (int rc = need(s, "scales")) return rc;
  if (int rc = aligned(U, 16, "U")) return rc;
  if (int rc = aligned(V, 16, "V")) return rc;
  if (int rc = aligned(y, 16, "y")) return rc;
  if (int rc = check_per_point(d, s)) return rc;
  MultTable mm;
  ShiftTable sh;
  double s_m;
  StageMults mu;
  if (int rc = contract_mults(p, s, &mm, &sh, &s_m)) return rc;
  if (int rc = output_mults(p, d, s, &mu, nullptr)) return rc;
  hipError_t e = launch_contract_output(p.g, p.two_brackets, (const int8_t*)U, (const int8_t*)V, y,
                                        p.m_bits, d->out_type, d->relu != 0, mu, mm,
                                        s->per_point ? &sh : nullptr, (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "contraction + output launch");
}

namespace {

// scale = float( max_ij( amax_ij * s_prev / (rho_i rho_j) ) / qmax ), 1 if everything is zero.
float scale_from(const unsigned long long* amax, const IMat& im, double s_prev, double qmax) {
  double best = 0.0;
  for (int i = 0; i < im.rows; ++i)
    for (int j = 0; j < im.rows; ++j) {
      const double real = ((double)amax[i * im.rows + j] * s_prev) / (double)(im.rho[i] * im.rho[j]);
      if (real > best) best = real;
    }
  return best > 0.0 ? (float)(best / qmax) : 1.0f;
}

// Per-point variant: out[ij] = float( amax_ij * s_prev / (rho_i rho_j) / qmax ), 1 where zero.
void scales_from_pt(const unsigned long long* amax, const IMat& im, double s_prev, double qmax,
                    float* out) {
  for (int i = 0; i < im.rows; ++i)
    for (int j = 0; j < im.rows; ++j) {
      const int q = i * im.rows + j;
      const double real = ((double)amax[q] * s_prev) / (double)(im.rho[i] * im.rho[j]);
      out[q] = real > 0.0 ? (float)(real / qmax) : 1.0f;
    }
}

struct CalCtx {
  hipStream_t st;
  unsigned long long* d_amax;
  unsigned long long h_amax[kMaxPts];
};

int cal_reset(CalCtx& c) {
  hipError_t e = hipMemsetAsync(c.d_amax, 0, sizeof c.h_amax, c.st);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "calibration memset");
}

int cal_read(CalCtx& c) {
  hipError_t e = hipMemcpyAsync(c.h_amax, c.d_amax, sizeof c.h_amax, hipMemcpyDeviceToHost, c.st);
  if (e == hipSuccess) e = hipStreamSynchronize(c.st);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "calibration read-back");
}

// One bracket: zero the maxima, run the calibration kernel, read them back.
int cal_bracket(CalCtx& c, int stage, const Plan& p, int phase, const void* in, int m_bits,
                const StageMults& mu, bool relu, const ShiftTable* sh = nullptr) {
  if (int rc = cal_reset(c)) return rc;
  hipError_t e = launch_calibrate_stage(stage, p.g, p.two_brackets, phase, in, m_bits, c.d_amax,
                                        mu, relu, sh, c.st);
  if (e != hipSuccess) return fail_hip(e, "calibration launch");
  return cal_read(c);
}

// s_m (and, per point, m_shift) from the exact int32 contraction result (U, V
// already in the workspace); leaves M computed with the chosen scales and
// reports what one unit fed to the output bracket stands for, and the shifts.
int calibrate_contraction(CalCtx& c, const wino_conv_desc_t* d, const wino_conv_desc_t& dd,
                          const Plan& p, const void* U, const void* V, void* M, void* M32,
                          wino_scales_t* s, double* s_fed, ShiftTable* sh) {
  const int n2 = (d->m + 2) * (d->m + 2);
  std::memset(sh, 0, sizeof *sh);
  MultTable unused;
  std::memset(&unused, 0, sizeof unused);
  if (p.m_bits == 32) {
    *s_fed = (double)s->s_u * (double)s->s_v;
    return wino_contract(&dd, U, V, M, s, c.st);
  }
  hipError_t e = launch_contract(p.g, (const int8_t*)U, (const int8_t*)V, M32, 32, unused, c.st);
  if (e != hipSuccess) return fail_hip(e, "contraction launch");
  if (int rc = cal_reset(c)) return rc;
  const long per_point_count = (long)p.g.T * d->K;
  e = s->per_point ? launch_absmax_i32((const int32_t*)M32, per_point_count, n2, c.d_amax, c.st)
                   : launch_absmax_i32((const int32_t*)M32, per_point_count * n2, 1, c.d_amax, c.st);
  if (e != hipSuccess) return fail_hip(e, "absmax launch");
  if (int rc = cal_read(c)) return rc;
  const double qm = p.m_bits == 8 ? 127.0 : 255.0;
  if (!s->per_point) {
    const double real = (double)c.h_amax[0] * ((double)s->s_u * (double)s->s_v);
    s->s_m = real > 0.0 ? (float)(real / qm) : 1.0f;
    *s_fed = (double)s->s_m;
  } else {
    double ideal[kMaxPts], top = 0.0;     // the scale that just covers point q
    for (int q = 0; q < n2; ++q) {
      ideal[q] = (double)c.h_amax[q] * ((double)s->s_u_pt[q] * (double)s->s_v_pt[q]) / qm;
      if (ideal[q] > top) top = ideal[q];
    }
    s->s_m = top > 0.0 ? (float)top : 1.0f;
    int smax = 0;
    for (int q = 0; q < n2; ++q) {
      int sft = 0;   // largest shift that does not clip the point
      while (sft < kMaxMShift && ideal[q] * std::ldexp(1.0, sft + 1) <= (double)s->s_m) ++sft;
      s->m_shift[q] = sft;
      if (sft > smax) smax = sft;
    }
    for (int q = 0; q < n2; ++q) sh->set(q, smax - s->m_shift[q]);
    *s_fed = std::ldexp((double)s->s_m, -smax);
  }
  return wino_contract(&dd, U, V, M, s, c.st);
}

size_t calibrate_layout(const wino_conv_desc_t* d, const Plan& p, size_t* oV, size_t* oU,
                        size_t* oM, size_t* oM32, size_t* oA) {
  const size_t n2 = (size_t)(d->m + 2) * (d->m + 2);
  size_t o = 0;
  *oV = o; o += round256(n2 * d->K * d->C);
  *oU = o; o += round256(n2 * p.g.T * d->C);
  *oM = o; o += round256(n2 * p.g.T * d->K * m_elem_bytes(p.m_bits));
  *oM32 = o; o += round256(n2 * p.g.T * d->K * 4);
  *oA = o; o += round256(sizeof(unsigned long long) * kMaxPts);
  return o;
}

}  // namespace

int wino_calibrate_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (!bytes) return fail(WINO_EINVAL, "null bytes");
  if (p.fp32) return fail(WINO_EUNSUPPORTED, "the fp32 path has no scales to calibrate");
  size_t a, b, c, e, f;
  *bytes = calibrate_layout(d, p, &a, &b, &c, &e, &f);
  return WINO_OK;
}

int wino_calibrate(const wino_conv_desc_t* d, const void* x, const void* w, void* y,
                   wino_scales_t* s, void* workspace, size_t ws_bytes, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (p.fp32) return fail(WINO_EUNSUPPORTED, "the fp32 path has no scales to calibrate");
  if (int rc = rows_only(p, "wino_calibrate")) return rc;
  if (int rc = legendre_only(p, "wino_calibrate")) return rc;
  if (d->C > kMaxChannelsExact)
    return fail(WINO_EOVERFLOW, "C = %d: calibration needs the exact int32 contraction result", d->C);
  if (int rc = need(s, "scales")) return rc;
  if (!good_scale(s->s_x) || !good_scale(s->s_w)) return fail(WINO_EINVAL, "s_x and s_w must be set");
  if (int rc = need(workspace, "workspace")) return rc;
  size_t oV, oU, oM, oM32, oA;
  const size_t want = calibrate_layout(d, p, &oV, &oU, &oM, &oM32, &oA);
  if (ws_bytes < want) return fail(WINO_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, want);
  if ((uintptr_t)workspace % 256) return fail(WINO_EWORKSPACE, "workspace must be 256-byte aligned");
  if (int rc = check_per_point(d, s)) return rc;
  const bool pp = s->per_point != 0;
  s->s_x1 = s->s_u = s->s_w1 = s->s_v = s->s_m = s->s_m1 = s->s_y = 1.0f;
  for (int q = 0; q < kMaxPts; ++q) {
    s->s_u_pt[q] = s->s_v_pt[q] = 1.0f;
    s->m_shift[q] = 0;
  }
  if (p.g.T == 0 || p.g.K == 0 || p.g.C == 0) return WINO_OK;
  if (int rc = need(x, "x")) return rc;
  if (int rc = need(w, "w")) return rc;
  char* ws = static_cast<char*>(workspace);
  void *V = ws + oV, *U = ws + oU, *M = ws + oM, *M32 = ws + oM32;
  CalCtx c{(hipStream_t)hip_stream, reinterpret_cast<unsigned long long*>(ws + oA), {}};
  wino_conv_desc_t dd = *d;
  dd.weights_pretransformed = 0;
  dd.fused = 0;
  StageMults mu;
  std::memset(&mu, 0, sizeof mu);

  // filters: s_w1 (Legendre inner bracket), s_v (one, or one per point)
  const IMat* w_outer = p.st.G;
  double w_prev = s->s_w;
  if (p.two_brackets) {
    if (int rc = cal_bracket(c, 0, p, 1, w, 8, mu, false)) return rc;
    s->s_w1 = scale_from(c.h_amax, *p.st.GP, s->s_w, 127.0);
    fill_mults(&mu.inner, *p.st.GP, s->s_w, s->s_w1);
    w_outer = p.st.Pinv;
    w_prev = s->s_w1;
  }
  if (int rc = cal_bracket(c, 0, p, 2, w, 8, mu, false)) return rc;
  if (pp)
    scales_from_pt(c.h_amax, *w_outer, w_prev, 127.0, s->s_v_pt);
  else
    s->s_v = scale_from(c.h_amax, *w_outer, w_prev, 127.0);
  if (int rc = wino_weight_transform(&dd, w, V, s, hip_stream)) return rc;

  // activations: s_x1 (Legendre inner bracket), s_u (one, or one per point)
  const IMat* x_outer = p.st.BT;
  double x_prev = s->s_x;
  if (p.two_brackets) {
    if (int rc = cal_bracket(c, 1, p, 1, x, 8, mu, false)) return rc;
    s->s_x1 = scale_from(c.h_amax, *p.st.PinvT, s->s_x, 127.0);
    fill_mults(&mu.inner, *p.st.PinvT, s->s_x, s->s_x1);
    x_outer = p.st.BPT;
    x_prev = s->s_x1;
  }
  if (int rc = cal_bracket(c, 1, p, 2, x, 8, mu, false)) return rc;
  if (pp)
    scales_from_pt(c.h_amax, *x_outer, x_prev, 127.0, s->s_u_pt);
  else
    s->s_u = scale_from(c.h_amax, *x_outer, x_prev, 127.0);
  if (int rc = wino_input_transform(&dd, x, U, s, hip_stream)) return rc;

  double s_m_eff;
  ShiftTable sh;
  if (int rc = calibrate_contraction(c, d, dd, p, U, V, M, M32, s, &s_m_eff, &sh)) return rc;
  const ShiftTable* shp = pp ? &sh : nullptr;

  // output: s_m1 (Legendre inner bracket), s_y
  if (p.two_brackets) {
    if (int rc = cal_bracket(c, 2, p, 1, M, p.m_bits, mu, false, shp)) return rc;
    s->s_m1 = scale_from(c.h_amax, *p.st.PinvT, s_m_eff, 127.0);
    fill_mults(&mu.inner, *p.st.PinvT, s_m_eff, s->s_m1);
    if (int rc = cal_bracket(c, 2, p, 2, M, p.m_bits, mu, d->relu != 0, shp)) return rc;
    s->s_y = scale_from(c.h_amax, *p.st.APT, s->s_m1, 127.0);
  } else {
    if (int rc = cal_bracket(c, 2, p, 2, M, p.m_bits, mu, d->relu != 0, shp)) return rc;
    s->s_y = scale_from(c.h_amax, *p.st.AT, s_m_eff, 127.0);
  }
  if (y)
    if (int rc = wino_output_transform(&dd, M, y, s, hip_stream)) return rc;
  return WINO_OK;
}

int wino_conv2d(const wino_conv_desc_t* d, const void* x, const void* w_or_V, void* y,
                const wino_scales_t* s, void* workspace, size_t ws_bytes, void* hip_stream) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (p.g.T == 0 || p.g.K == 0) return WINO_OK;   // no output element exists
  if (int rc = check_per_point(d, s)) return rc;
  Path path;
  if (int rc = select_path(d, p, &path)) return rc;
  bool frag;
  if (int rc = conv_layout(d, p, path, &frag)) return rc;
  size_t want = 0;
  if (int rc = wino_workspace_bytes(d, &want)) return rc;
  wino_conv_desc_t dsel = *d;
  dsel.fused = path == kPathFusedAll;
  dsel.operand_layout = frag ? WINO_LAYOUT_FRAGMENTS : WINO_LAYOUT_ROWS;
  d = &dsel;
  if (int rc = need(workspace, "workspace")) return rc;
  if (ws_bytes < want) return fail(WINO_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, want);
  if ((uintptr_t)workspace % 256) return fail(WINO_EWORKSPACE, "workspace must be 256-byte aligned");
  char* ws = static_cast<char*>(workspace);
  const void* V = w_or_V;
  void* Vws = nullptr;
  if (!d->weights_pretransformed) {
    Vws = ws;
    V = ws;
    ws += round256(v_bytes_of(p, frag));
    // the fused variant transforms the filters on their own; the split path
    // does it together with the input transform, in one launch (below)
    if (d->fused)
      if (int rc = wino_weight_transform(d, w_or_V, Vws, s, hip_stream)) return rc;
  }
  if (d->fused) {
    if (int rc = need(x, "x")) return rc;
    if (int rc = need(y, "y")) return rc;
    if (int rc = need(s, "scales")) return rc;
    if (int rc = aligned(V, 16, "V")) return rc;
    StageMults in_mu, out_mu;
    MultTable m_mult;
    ShiftTable sh;
    double s_m;
    if (int rc = input_mults(p, s, &in_mu)) return rc;
    if (int rc = contract_mults(p, s, &m_mult, &sh, &s_m)) return rc;
    if (int rc = output_mults(p, d, s, &out_mu, nullptr)) return rc;
    hipError_t e = launch_fused(p.g, p.two_brackets, (const int8_t*)x, (const int8_t*)V, y,
                                p.m_bits, d->out_type, d->relu != 0, in_mu, out_mu, m_mult,
                                s->per_point ? &sh : nullptr, (hipStream_t)hip_stream);
    return e == hipSuccess ? WINO_OK : fail_hip(e, "fused launch");
  }
  void* U = ws;
  ws += round256(u_bytes_of(p, frag));
  void* M = ws;
  if (Vws) {
    if (int rc = wino_transform_operands(d, x, U, w_or_V, Vws, s, hip_stream)) return rc;
  } else {
    if (int rc = wino_input_transform(d, x, U, s, hip_stream)) return rc;
  }
  if (path == kPathConOut) return wino_contract_output(d, U, V, y, s, hip_stream);
  if (int rc = wino_contract(d, U, V, M, s, hip_stream)) return rc;
  return wino_output_transform(d, M, y, s, hip_stream);
}

// ---------------------------------------------------------------------------
// Flex layer: run-time fp32 matrices in the G_P / B_P / A_P brackets.
// ---------------------------------------------------------------------------
namespace {

struct FlexPlan {
  Plan p;
  FlexMats fm;
};

int make_flex_plan(const wino_conv_desc_t* d, const wino_flex_matrices_t* f, FlexPlan* fp) {
  if (int rc = make_plan(d, &fp->p)) return rc;
  const Plan& p = fp->p;
  if (p.fp32) return fail(WINO_EUNSUPPORTED, "flex layers run on the int8 path (bits_in = 8)");
  if (int rc = rows_only(p, "a flex call")) return rc;
  if (p.legendre && d->base != WINO_BASE_LEGENDRE)
    return fail(WINO_EUNSUPPORTED, "flex layers are built for the canonical and the Legendre base");
  if (p.legendre && !p.two_brackets)
    return fail(WINO_EUNSUPPORTED, "a flex layer in the Legendre base needs inner_quant = 1 "
                                   "(run-time matrices cannot be multiplied out with P^{-1})");
  if (d->out_type == WINO_OUT_I32)
    return fail(WINO_EUNSUPPORTED, "a flex layer has fp32 or int8 output");
  if (d->fused == WINO_FUSED_ON)
    return fail(WINO_EUNSUPPORTED, "the fused variant has no flex form");
  if (!f || !f->GP || !f->BPT || !f->APT) return fail(WINO_EINVAL, "null flex matrix");
  const int n = d->m + 2;
  std::memset(&fp->fm, 0, sizeof fp->fm);
  struct { const float* src; float* dst; int count; const char* name; } parts[3] = {
      {f->GP, fp->fm.GP, n * 3, "GP"}, {f->BPT, fp->fm.BPT, n * n, "BPT"},
      {f->APT, fp->fm.APT, d->m * n, "APT"}};
  for (auto& part : parts)
    for (int i = 0; i < part.count; ++i) {
      const float v = part.src[i];
      if (!std::isfinite(v) || std::fabs(v) > 1048576.0f)
        return fail(WINO_EINVAL, "flex matrix %s[%d] = %g: entries must be finite and at most 2^20 "
                                 "in magnitude", part.name, i, (double)v);
      part.dst[i] = v;
    }
  return WINO_OK;
}

// Multipliers of the three flex stages.  `first` is the cast after the fp32
// bracket; the integer P^{-1} brackets use the tables of the static path.
int flex_no_per_point(const wino_scales_t* s) {
  return s->per_point ? fail(WINO_EUNSUPPORTED, "the flex calls take per-tensor scales") : WINO_OK;
}

int flex_weight_mults(const Plan& p, const wino_scales_t* s, StageMults* mu, float* first) {
  if (int rc = flex_no_per_point(s)) return rc;
  std::memset(mu, 0, sizeof *mu);
  if (!good_scale(s->s_w) || !good_scale(s->s_v)) return fail(WINO_EINVAL, "bad s_w / s_v");
  if (p.two_brackets) {
    if (!good_scale(s->s_w1)) return fail(WINO_EINVAL, "bad s_w1");
    *first = (float)((double)s->s_w / (double)s->s_w1);
    fill_mults(&mu->outer, *p.st.Pinv, s->s_w1, s->s_v);
  } else {
    *first = (float)((double)s->s_w / (double)s->s_v);
  }
  return WINO_OK;
}

int flex_input_mults(const Plan& p, const wino_scales_t* s, StageMults* mu, float* mult_u) {
  if (int rc = flex_no_per_point(s)) return rc;
  std::memset(mu, 0, sizeof *mu);
  if (!good_scale(s->s_x) || !good_scale(s->s_u)) return fail(WINO_EINVAL, "bad s_x / s_u");
  if (p.two_brackets) {
    if (!good_scale(s->s_x1)) return fail(WINO_EINVAL, "bad s_x1");
    fill_mults(&mu->inner, *p.st.PinvT, s->s_x, s->s_x1);
    *mult_u = (float)((double)s->s_x1 / (double)s->s_u);
  } else {
    *mult_u = (float)((double)s->s_x / (double)s->s_u);
  }
  return WINO_OK;
}

int flex_output_mults(const Plan& p, const wino_conv_desc_t* d, const wino_scales_t* s,
                      StageMults* mu, float* mult_out) {
  if (int rc = flex_no_per_point(s)) return rc;
  std::memset(mu, 0, sizeof *mu);
  MultTable dummy;
  double s_prev;
  if (int rc = contract_mults(p, s, &dummy, nullptr, &s_prev)) return rc;
  if (p.two_brackets) {
    if (!good_scale(s->s_m1)) return fail(WINO_EINVAL, "bad s_m1");
    fill_mults(&mu->inner, *p.st.PinvT, s_prev, s->s_m1);
    s_prev = (double)s->s_m1;
  }
  if (d->out_type == WINO_OUT_I8) {
    if (!good_scale(s->s_y)) return fail(WINO_EINVAL, "bad s_y");
    *mult_out = (float)(s_prev / (double)s->s_y);
  } else {
    *mult_out = (float)s_prev;
  }
  return WINO_OK;
}

// scale = float( max |fp32 bracket value| * s_prev / qmax ), 1 if everything is zero.
float flex_scale_from(unsigned long long amax_bits, double s_prev, double qmax) {
  const uint32_t bits = (uint32_t)amax_bits;
  float amax;
  std::memcpy(&amax, &bits, sizeof amax);
  const double real = (double)amax * s_prev;
  return real > 0.0 ? (float)(real / qmax) : 1.0f;
}

int flex_cal_launch(CalCtx& c, int stage, const FlexPlan& fp, int mode, const void* in,
                    const StageMults& mu, float mult, bool relu) {
  if (int rc = cal_reset(c)) return rc;
  hipError_t e = launch_flex_stage(stage, fp.p.g, fp.p.two_brackets, mode, in, fp.p.m_bits, nullptr,
                                   0, relu, c.d_amax, fp.fm, mu, mult, c.st);
  if (e != hipSuccess) return fail_hip(e, "flex calibration launch");
  return cal_read(c);
}

}  // namespace

int wino_flex_weight_transform(const wino_conv_desc_t* d, const wino_flex_matrices_t* f,
                               const void* w, void* V, const wino_scales_t* s, void* hip_stream) {
  FlexPlan fp;
  if (int rc = make_flex_plan(d, f, &fp)) return rc;
  if ((long)fp.p.g.K * fp.p.g.C == 0) return WINO_OK;
  if (int rc = need(w, "w")) return rc;
  if (int rc = need(V, "V")) return rc;
  if (int rc = need(s, "scales")) return rc;
  StageMults mu;
  float first;
  if (int rc = flex_weight_mults(fp.p, s, &mu, &first)) return rc;
  hipError_t e = launch_flex_stage(0, fp.p.g, fp.p.two_brackets, 0, w, 8, V, 0, false, nullptr,
                                   fp.fm, mu, first, (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "flex weight transform launch");
}

int wino_flex_input_transform(const wino_conv_desc_t* d, const wino_flex_matrices_t* f,
                              const void* x, void* U, const wino_scales_t* s, void* hip_stream) {
  FlexPlan fp;
  if (int rc = make_flex_plan(d, f, &fp)) return rc;
  if ((long)fp.p.g.T * fp.p.g.C == 0) return WINO_OK;
  if (int rc = need(x, "x")) return rc;
  if (int rc = need(U, "U")) return rc;
  if (int rc = need(s, "scales")) return rc;
  StageMults mu;
  float mult_u;
  if (int rc = flex_input_mults(fp.p, s, &mu, &mult_u)) return rc;
  hipError_t e = launch_flex_stage(1, fp.p.g, fp.p.two_brackets, 0, x, 8, U, 0, false, nullptr,
                                   fp.fm, mu, mult_u, (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "flex input transform launch");
}

int wino_flex_output_transform(const wino_conv_desc_t* d, const wino_flex_matrices_t* f,
                               const void* M, void* y, const wino_scales_t* s, void* hip_stream) {
  FlexPlan fp;
  if (int rc = make_flex_plan(d, f, &fp)) return rc;
  if ((long)fp.p.g.T * fp.p.g.K == 0) return WINO_OK;
  if (int rc = need(M, "M")) return rc;
  if (int rc = need(y, "y")) return rc;
  if (int rc = need(s, "scales")) return rc;
  StageMults mu;
  float mult_out;
  if (int rc = flex_output_mults(fp.p, d, s, &mu, &mult_out)) return rc;
  hipError_t e = launch_flex_stage(2, fp.p.g, fp.p.two_brackets, 0, M, fp.p.m_bits, y, d->out_type,
                                   d->relu != 0, nullptr, fp.fm, mu, mult_out,
                                   (hipStream_t)hip_stream);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "flex output transform launch");
}

int wino_flex_conv2d(const wino_conv_desc_t* d, const wino_flex_matrices_t* f, const void* x,
                     const void* w_or_V, void* y, const wino_scales_t* s, void* workspace,
                     size_t ws_bytes, void* hip_stream) {
  FlexPlan fp;
  if (int rc = make_flex_plan(d, f, &fp)) return rc;
  const Plan& p = fp.p;
  if (p.g.T == 0 || p.g.K == 0) return WINO_OK;   // no output element exists
  wino_conv_desc_t dd = *d;
  dd.fused = WINO_FUSED_OFF;
  size_t want = 0;
  if (int rc = wino_workspace_bytes(&dd, &want)) return rc;
  if (int rc = need(workspace, "workspace")) return rc;
  if (ws_bytes < want) return fail(WINO_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, want);
  if ((uintptr_t)workspace % 256) return fail(WINO_EWORKSPACE, "workspace must be 256-byte aligned");
  const size_t n2 = (size_t)(d->m + 2) * (d->m + 2);
  char* ws = static_cast<char*>(workspace);
  const void* V = w_or_V;
  void* Vws = nullptr;
  if (!d->weights_pretransformed) {
    Vws = ws;
    V = ws;
    ws += round256(n2 * d->K * d->C);
  }
  void* U = ws;
  ws += round256(n2 * p.g.T * d->C);
  void* M = ws;
  if (Vws && (long)p.g.T * p.g.C && (long)p.g.K * p.g.C) {
    // both operand transforms are independent: one launch
    if (int rc = need(x, "x")) return rc;
    if (int rc = need(w_or_V, "w")) return rc;
    if (int rc = need(s, "scales")) return rc;
    StageMults mu_in, mu_w;
    float mult_u, mult_first;
    if (int rc = flex_input_mults(p, s, &mu_in, &mult_u)) return rc;
    if (int rc = flex_weight_mults(p, s, &mu_w, &mult_first)) return rc;
    hipError_t e = launch_flex_operands(p.g, p.two_brackets, (const int8_t*)x, (int8_t*)U,
                                        (const int8_t*)w_or_V, (int8_t*)Vws, fp.fm, mu_in, mult_u,
                                        mu_w, mult_first, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail_hip(e, "flex operand-transform launch");
  } else {
    if (Vws)
      if (int rc = wino_flex_weight_transform(&dd, f, w_or_V, Vws, s, hip_stream)) return rc;
    if (int rc = wino_flex_input_transform(&dd, f, x, U, s, hip_stream)) return rc;
  }
  if (int rc = wino_contract(&dd, U, V, M, s, hip_stream)) return rc;
  return wino_flex_output_transform(&dd, f, M, y, s, hip_stream);
}

int wino_flex_calibrate(const wino_conv_desc_t* d, const wino_flex_matrices_t* f, const void* x,
                        const void* w, void* y, wino_scales_t* s, void* workspace,
                        size_t ws_bytes, void* hip_stream) {
  FlexPlan fp;
  if (int rc = make_flex_plan(d, f, &fp)) return rc;
  const Plan& p = fp.p;
  if (d->C > kMaxChannelsExact)
    return fail(WINO_EOVERFLOW, "C = %d: calibration needs the exact int32 contraction result", d->C);
  if (int rc = need(s, "scales")) return rc;
  if (!good_scale(s->s_x) || !good_scale(s->s_w)) return fail(WINO_EINVAL, "s_x and s_w must be set");
  if (int rc = flex_no_per_point(s)) return rc;
  if (int rc = need(workspace, "workspace")) return rc;
  size_t oV, oU, oM, oM32, oA;
  const size_t want = calibrate_layout(d, p, &oV, &oU, &oM, &oM32, &oA);
  if (ws_bytes < want) return fail(WINO_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, want);
  if ((uintptr_t)workspace % 256) return fail(WINO_EWORKSPACE, "workspace must be 256-byte aligned");
  s->s_x1 = s->s_u = s->s_w1 = s->s_v = s->s_m = s->s_m1 = s->s_y = 1.0f;
  if (p.g.T == 0 || p.g.K == 0 || p.g.C == 0) return WINO_OK;
  if (int rc = need(x, "x")) return rc;
  if (int rc = need(w, "w")) return rc;
  char* ws = static_cast<char*>(workspace);
  void *V = ws + oV, *U = ws + oU, *M = ws + oM, *M32 = ws + oM32;
  CalCtx c{(hipStream_t)hip_stream, reinterpret_cast<unsigned long long*>(ws + oA), {}};
  wino_conv_desc_t dd = *d;
  dd.weights_pretransformed = 0;
  dd.fused = 0;
  StageMults mu;
  std::memset(&mu, 0, sizeof mu);

  // filters: the fp32 G bracket first, then (Legendre) the integer P^{-1} bracket
  if (int rc = flex_cal_launch(c, 0, fp, 1, w, mu, 1.f, false)) return rc;
  if (p.two_brackets) {
    s->s_w1 = flex_scale_from(c.h_amax[0], s->s_w, 127.0);
    const float first = (float)((double)s->s_w / (double)s->s_w1);
    if (int rc = flex_cal_launch(c, 0, fp, 2, w, mu, first, false)) return rc;
    s->s_v = scale_from(c.h_amax, *p.st.Pinv, s->s_w1, 127.0);
  } else {
    s->s_v = flex_scale_from(c.h_amax[0], s->s_w, 127.0);
  }
  if (int rc = wino_flex_weight_transform(&dd, f, w, V, s, hip_stream)) return rc;

  // activations: (Legendre) the integer P^{-T} bracket, then the fp32 B bracket
  double s_prev = s->s_x;
  if (p.two_brackets) {
    if (int rc = cal_bracket(c, 1, p, 1, x, 8, mu, false)) return rc;
    s->s_x1 = scale_from(c.h_amax, *p.st.PinvT, s->s_x, 127.0);
    fill_mults(&mu.inner, *p.st.PinvT, s->s_x, s->s_x1);
    s_prev = s->s_x1;
  }
  if (int rc = flex_cal_launch(c, 1, fp, 1, x, mu, 1.f, false)) return rc;
  s->s_u = flex_scale_from(c.h_amax[0], s_prev, 127.0);
  if (int rc = wino_flex_input_transform(&dd, f, x, U, s, hip_stream)) return rc;

  double s_m_eff;
  ShiftTable sh_unused;
  if (int rc = calibrate_contraction(c, d, dd, p, U, V, M, M32, s, &s_m_eff, &sh_unused)) return rc;

  // output: (Legendre) the integer P^{-T} bracket, then the fp32 A bracket
  s_prev = s_m_eff;
  if (p.two_brackets) {
    if (int rc = cal_bracket(c, 2, p, 1, M, p.m_bits, mu, false)) return rc;
    s->s_m1 = scale_from(c.h_amax, *p.st.PinvT, s_m_eff, 127.0);
    fill_mults(&mu.inner, *p.st.PinvT, s_m_eff, s->s_m1);
    s_prev = s->s_m1;
  }
  if (int rc = flex_cal_launch(c, 2, fp, 1, M, mu, 1.f, d->relu != 0)) return rc;
  s->s_y = flex_scale_from(c.h_amax[0], s_prev, 127.0);
  if (y)
    if (int rc = wino_flex_output_transform(&dd, f, M, y, s, hip_stream)) return rc;
  return WINO_OK;
}

namespace {
struct FlexBwdLayout {
  size_t dM, dU, dV, dXt, part_out, part_in, part_w, total;
  long out_blocks, in_blocks, w_blocks;
};
FlexBwdLayout flex_bwd_layout(const Geometry& g) {
  const size_t n2 = (size_t)(g.m + 2) * (g.m + 2);
  const size_t T = (size_t)g.T, C = (size_t)g.C, K = (size_t)g.K;
  FlexBwdLayout l;
  l.out_blocks = (long)((T * K + 255) / 256);
  l.in_blocks = (long)((T * C + 255) / 256);
  l.w_blocks = (long)((K * C + 255) / 256);
  size_t o = 0;
  l.dM = o;  o += round256(n2 * T * K * 4);
  l.dU = o;  o += round256(n2 * T * C * 4);
  l.dV = o;  o += round256((size_t)backward_dv_splits(g) * n2 * K * C * 4);
  l.dXt = o; o += round256(n2 * T * C * 4);
  l.part_out = o; o += (size_t)l.out_blocks * 256;
  l.part_in = o;  o += (size_t)l.in_blocks * 256;
  l.part_w = o;   o += (size_t)l.w_blocks * 256;
  l.total = o;
  return l;
}
}  // namespace

int wino_flex_backward_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes) {
  Plan p;
  if (int rc = make_plan(d, &p)) return rc;
  if (p.fp32) return fail(WINO_EUNSUPPORTED, "flex layers run on the int8 path (bits_in = 8)");
  if (int rc = rows_only(p, "a flex call")) return rc;
  if (p.legendre && d->base != WINO_BASE_LEGENDRE)
    return fail(WINO_EUNSUPPORTED, "flex layers are built for the canonical and the Legendre base");
  if (!bytes) return fail(WINO_EINVAL, "null bytes");
  *bytes = flex_bwd_layout(p.g).total;
  if (*bytes == 0) *bytes = 256;
  return WINO_OK;
}

int wino_flex_backward(const wino_conv_desc_t* d, const wino_flex_matrices_t* f, const void* dy,
                       const void* x, const void* w, const void* U, const void* V, const void* M,
                       const wino_scales_t* s, void* dx, void* dw, const wino_flex_grads_t* grads,
                       void* workspace, size_t ws_bytes, void* hip_stream) {
  FlexPlan fp;
  if (int rc = make_flex_plan(d, f, &fp)) return rc;
  const Plan& p = fp.p;
  const Geometry& g = p.g;
  if (g.N <= 0 || g.H <= 0 || g.W <= 0 || g.C <= 0 || g.K <= 0)
    return fail(WINO_EINVAL, "the flex backward pass needs positive dimensions");
  if (int rc = need(s, "scales")) return rc;
  if (!grads || !grads->dGP || !grads->dBPT || !grads->dAPT)
    return fail(WINO_EINVAL, "null matrix gradient");
  const struct { const void* ptr; const char* name; } ptrs[] = {
      {dy, "dy"}, {x, "x"}, {w, "w"}, {U, "U"}, {V, "V"}, {M, "M"}, {dx, "dx"}, {dw, "dw"}};
  for (const auto& q : ptrs)
    if (int rc = need(q.ptr, q.name)) return rc;
  for (const auto& q : {ptrs[0], ptrs[3], ptrs[4]})
    if (int rc = aligned(q.ptr, 16, q.name)) return rc;
  StageMults mu_in, mu_out;
  float mult_unused, s_in_m;
  if (int rc = flex_input_mults(p, s, &mu_in, &mult_unused)) return rc;
  wino_conv_desc_t dreal = *d;
  dreal.out_type = WINO_OUT_F32;          // asks flex_output_mults for the scale of the A_P bracket's input
  if (int rc = flex_output_mults(p, &dreal, s, &mu_out, &s_in_m)) return rc;
  if (!good_scale(s->s_w)) return fail(WINO_EINVAL, "bad s_w");
  const float s_in_x = p.two_brackets ? s->s_x1 : s->s_x;
  const FlexBwdLayout l = flex_bwd_layout(g);
  if (int rc = need(workspace, "workspace")) return rc;
  if (ws_bytes < l.total) return fail(WINO_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, l.total);
  if ((uintptr_t)workspace % 256) return fail(WINO_EWORKSPACE, "workspace must be 256-byte aligned");
  char* ws = static_cast<char*>(workspace);
  float* dM = reinterpret_cast<float*>(ws + l.dM);
  float* dU = reinterpret_cast<float*>(ws + l.dU);
  float* dV = reinterpret_cast<float*>(ws + l.dV);
  float* dXt = reinterpret_cast<float*>(ws + l.dXt);
  float* part_out = reinterpret_cast<float*>(ws + l.part_out);
  float* part_in = reinterpret_cast<float*>(ws + l.part_in);
  float* part_w = reinterpret_cast<float*>(ws + l.part_w);
  const int n = g.m + 2, n2 = n * n;
  MultTable su, sv;
  std::memset(&su, 0, sizeof su);
  std::memset(&sv, 0, sizeof sv);
  for (int q = 0; q < n2; ++q) su.v[q] = s->s_u, sv.v[q] = s->s_v;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e = launch_flex_backward_output(g, p.legendre, M, p.m_bits, (const float*)dy, dM,
                                             part_out, fp.fm, mu_out, s_in_m, st);
  if (e != hipSuccess) return fail_hip(e, "flex backward output-bracket launch");
  e = launch_backward_gemms(g, dM, (const int8_t*)U, (const int8_t*)V, dU, dV, su, sv, st);
  if (e != hipSuccess) return fail_hip(e, "flex backward contraction launch");
  e = launch_backward_sum_splits(g, dV, st);            // no launch unless dV came in several parts
  if (e != hipSuccess) return fail_hip(e, "flex backward partial-sum launch");
  e = launch_flex_backward_input_weight(g, p.legendre, (const int8_t*)x, dU, dXt, part_in,
                                        (const int8_t*)w, dV, (float*)dw, part_w, fp.fm, mu_in,
                                        s_in_x, s->s_w, st);
  if (e != hipSuccess) return fail_hip(e, "flex backward input / filter bracket launch");
  e = launch_flex_backward_tile_sum(g, dXt, (float*)dx, st);
  if (e != hipSuccess) return fail_hip(e, "flex backward tile-sum launch");
  const float* const parts[3] = {part_out, part_in, part_w};
  const long part_rows[3] = {l.out_blocks, l.in_blocks, l.w_blocks};
  const int part_counts[3] = {g.m * n, n2, n * 3};
  float* const sums[3] = {(float*)grads->dAPT, (float*)grads->dBPT, (float*)grads->dGP};
  e = launch_sum_partials(parts, part_rows, part_counts, sums, st);
  return e == hipSuccess ? WINO_OK : fail_hip(e, "flex backward matrix-gradient launch");
}

}  // extern "C"
