/* wino.h -- C ABI of libwino: quantised Winograd/Toom-Cook 2-D convolution
 * (3x3, stride 1, pad 1) with transforms in the canonical or monic-Legendre
 * polynomial base, for AMD MI355X (gfx950).
 *
 * Conventions
 *   m = output tile edge, r = kernel edge (3), n = m + r - 1 = Winograd tile
 *   edge, TH = ceil(H/m), TW = ceil(W/m), T = N*TH*TW tiles, tile index
 *   t = (b*TH + ty)*TW + tx, Winograd point p = i*n + j.
 *   Device tensors (all dense, row-major in the order written):
 *     x [N][H][W][C] int8      activations, NHWC
 *     w [K][C][3][3] int8      filters, KCRS
 *     V [n*n][K][C]  int8      transformed filters
 *     U [n*n][T][C]  int8      transformed input tiles
 *     M [n*n][T][K]  int8 (bits_hadamard 8) | int16 (9) | int32 (32)
 *     y [N][H][W][K] float | int8 | int32 (see out_type)
 *   A stored code q of a tensor with scale s stands for the real value q*s.
 *   Every device tensor must start on a 16-byte boundary (EINVAL otherwise).
 *
 * Every function returns WINO_OK (0) or a negative error code and never
 * throws or aborts; wino_last_error() gives the text of the last failure on
 * the calling thread.  Functions taking a stream are asynchronous on it,
 * allocate nothing and never synchronise; all device buffers, the workspace
 * included, are owned by the caller.
 */
#ifndef WINO_H
#define WINO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  WINO_OK = 0,
  WINO_EINVAL = -1,       /* bad argument, shape, duplicate point, null pointer */
  WINO_EUNSUPPORTED = -2, /* (m, r), bits or option combination not built       */
  WINO_EOVERFLOW = -3,    /* rational or integer-stage bound exceeded           */
  WINO_EWORKSPACE = -4,   /* workspace too small or misaligned                  */
  WINO_EHIP = -5          /* HIP runtime error, text in wino_last_error()       */
};

enum {
  WINO_BASE_CANONICAL = 0,
  WINO_BASE_LEGENDRE = 1,
  WINO_BASE_CHEBYSHEV = 2, /* monic Chebyshev polynomials (first kind)    */
  WINO_BASE_HERMITE = 3    /* monic Hermite polynomials (probabilists')   */
};
enum { WINO_OUT_F32 = 0, WINO_OUT_I32 = 1, WINO_OUT_I8 = 2 };
enum { WINO_FUSED_OFF = 0, WINO_FUSED_ON = 1, WINO_FUSED_AUTO = 2 };
/* Memory order of the transformed operands U and V (int8 path).
 * ROWS: U [n*n][T][C], V [n*n][K][C], as written under "Conventions".
 * FRAGMENTS: the register layout of the 16x16x64 int8 matrix instruction, so
 * that the kernel that contracts them loads them without any rearrangement:
 * rows (tiles of U, output channels of V) in groups of 16, channels in chunks
 * of 64, each 16 x 64 block one contiguous KiB ordered [c%64/16][row%16][c%16]:
 *   offset(p, row, c) = ((p*RG + row/16)*NCH + c/64)*1024
 *                       + (c%64/16)*256 + (row%16)*16 + c%16,
 *   RG = ceil(rows/16), NCH = ceil(C/64); size n*n*RG*NCH KiB
 *   (wino_operand_bytes).  Rows past the last one are never written; channels
 * past C are zeros in V.  Written by the three operand-transform calls, read by
 * wino_contract_output and by wino_conv2d (a pretransformed V); every other
 * call takes ROWS only (EUNSUPPORTED otherwise). */
enum { WINO_LAYOUT_ROWS = 0, WINO_LAYOUT_FRAGMENTS = 1 };
enum {
  WINO_MAT_G = 0,     /* n x r  Section 3: filter transform                    */
  WINO_MAT_BT = 1,    /* n x n  Section 3: input transform                     */
  WINO_MAT_AT = 2,    /* m x n  Section 3: output transform                    */
  WINO_MAT_PT = 3,    /* n x n  Section 4.1: base change P^T                   */
  WINO_MAT_PINVT = 4, /* n x n  Section 4.1: P^{-T}                            */
  WINO_MAT_GP = 5,    /* n x r  G_P = P G                                      */
  WINO_MAT_BPT = 6,   /* n x n  B_P^T = (P B)^T                                */
  WINO_MAT_APT = 7    /* m x n  A_P^T = (P A)^T                                */
};

typedef struct { int64_t num, den; } wino_rat_t;   /* den > 0, reduced */
typedef struct wino_matrices wino_matrices_t;      /* opaque, host memory */

/* Section 3 ("Winograd algorithm") and Section 4.1: exact rational Toom-Cook
 * matrices G, B^T, A^T for F(m, r) from `n_finite` = m+r-2 distinct finite
 * points (host array; the point at infinity is implicit and last), plus the
 * base-change factors P^T, P^{-T} and G_P = P G, B_P = P B, A_P = P A.
 * base = WINO_BASE_LEGENDRE: P^T rows are the monic Legendre polynomials;
 * WINO_BASE_CHEBYSHEV / WINO_BASE_HERMITE: the monic Chebyshev (first kind) /
 * Hermite (probabilists') polynomials, the alternatives Section 4.1 names;
 * base = WINO_BASE_CANONICAL: P = I.  m+r-1 <= 8.
 * On success *out owns a host handle to be released with wino_free_matrices.
 * Errors: EINVAL (null, sizes, zero denominator, duplicate point),
 * EUNSUPPORTED (m+r-1 > 8), EOVERFLOW (an int64 rational overflowed). */
int wino_make_matrices(int m, int r, const wino_rat_t* points, int n_finite, int base,
                       wino_matrices_t** out);
void wino_free_matrices(wino_matrices_t* h);

/* Copies matrix `which` (WINO_MAT_*) row-major into host buffer `buf`
 * (room for 64 entries is always enough) and reports its shape. */
int wino_get_matrix(const wino_matrices_t* h, int which, wino_rat_t* buf, int* rows, int* cols);

/* Integer form used by the quantised stages: matrix = diag(1/row_lcd) * N with
 * row_lcd[i] the least common denominator of row i.  N: rows*cols int64
 * row-major, row_lcd: rows int64, both host buffers. */
int wino_get_int_form(const wino_matrices_t* h, int which, int64_t* N, int64_t* row_lcd,
                      int* rows, int* cols);

typedef struct {
  int N, H, W, C, K;          /* C and K multiples of 16                          */
  int m, r;                   /* (2,3), (4,3) or (6,3); standard point sets
                                 {0,1,-1}, {0,1,-1,2,-2}, {0,1,-1,2,-2,1/2,-1/2}  */
  int base;                   /* WINO_BASE_*.  Chebyshev and Hermite (the other
                                 bases Section 4.1 names; eq. 4 with their P):
                                 the four stage calls, wino_transform_operands
                                 and wino_conv2d with one kernel per stage,
                                 int8 path, per-tensor scales; every other call
                                 and variant is EUNSUPPORTED for them             */
  int bits_in;                /* 8: int8 path; 32: fp32 path without any cast: x, w,
                                 U, V, M, y are float in the same layouts, scales
                                 are ignored (may be null), output is fp32        */
  int bits_hadamard;          /* 8 | 9 | 32: width kept for the contraction result
                                 (Section 5: the Hadamard stage kept on 9 bits)   */
  int inner_quant;            /* Legendre only: casts on the inner brackets of
                                 eq. 4 (1) or brackets multiplied out (0)         */
  int out_type;               /* WINO_OUT_*; I32 needs an integer A^T (canonical
                                 base, m = 2 or 4)                                */
  int relu;                   /* clamp the output at zero                         */
  int weights_pretransformed; /* wino_conv2d: second pointer is V, not w          */
  int fused;                  /* wino_conv2d: WINO_FUSED_*: OFF = one kernel per
                                 stage (V, U, M all in the workspace).  ON = the
                                 contraction result M never leaves the chip: one
                                 kernel for the whole layer where C <= 64 and
                                 m = 2 or 4 (U stays on chip too), otherwise the
                                 input transform followed by ONE kernel for
                                 contraction + output transform (U in the
                                 workspace); needs bits_hadamard 8 or 9 and fp32
                                 or int8 output.  AUTO = the fastest of the three
                                 for the shape, as measured: the single kernel for
                                 C, K <= 64; the two-kernel form (m = 2 or 4) for
                                 layers with C <= 128, for layers with C <= 256
                                 whose M is 9 bits wide or whose grid is about
                                 one work group per compute unit, and whenever V
                                 is handed over in fragment order; one kernel per
                                 stage for the rest                               */
  int operand_layout;         /* WINO_LAYOUT_*: order of U and V in the stage
                                 calls that write or read them; in wino_conv2d
                                 the order of a pretransformed V (U, and a V it
                                 computes itself, live in the workspace in the
                                 order its kernels want).  The two-kernel form
                                 is fast with FRAGMENTS; given a pretransformed
                                 V in ROWS, AUTO runs one kernel per stage; given
                                 one in FRAGMENTS it runs the two-kernel form
                                 (wino_preferred_operand_layout says which of
                                 the two is the faster for a layer)               */
} wino_conv_desc_t;

/* Symmetric scales, supplied by the caller (or chosen by wino_calibrate).
 * s_x1, s_w1, s_m1 belong to the inner brackets of eq. 4 and are ignored for
 * the canonical base or inner_quant = 0; s_m is ignored for bits_hadamard = 32;
 * s_y only matters for I8 output.
 *
 * per_point = 0: one scale per tensor (the paper's setting).
 * per_point = 1 (an option of this library, not in the paper): the three
 * Winograd-domain tensors around the Hadamard stage get one scale per point
 * p = i*n + j, because their value ranges differ by orders of magnitude from
 * point to point:  U[p] has scale s_u_pt[p], V[p] has scale s_v_pt[p] (s_u, s_v
 * are then ignored), and M[p] has scale s_m / 2^m_shift[p] with
 * 0 <= m_shift[p] <= WINO_MAX_M_SHIFT.  The powers of two keep the output
 * bracket in exact integers: it is fed with code << (smax - m_shift[p]) at the
 * common scale s_m / 2^smax, smax = max_p m_shift[p].  Needs bits_hadamard 8 or
 * 9 and F32 or I8 output; not available in the flex calls.  Only the first
 * n*n entries of the arrays are read. */
enum { WINO_MAX_M_SHIFT = 8 };
typedef struct {
  float s_x, s_x1, s_u, s_w, s_w1, s_v, s_m, s_m1, s_y;
  int per_point;
  float s_u_pt[64];
  float s_v_pt[64];
  int m_shift[64];
} wino_scales_t;

/* Bytes of V and of U (host pointers, either may be null) in the order
 * d->operand_layout names. */
int wino_operand_bytes(const wino_conv_desc_t* d, size_t* v_bytes, size_t* u_bytes);

/* *layout (host) = the order in which wino_conv2d runs this layer fastest when
 * it is handed a pretransformed V: FRAGMENTS where AUTO would take the
 * two-kernel form, ROWS otherwise (d->operand_layout itself is ignored). */
int wino_preferred_operand_layout(const wino_conv_desc_t* d, int* layout);

/* Bytes of device workspace wino_conv2d needs for this descriptor: V unless
 * pretransformed, U unless the single-kernel variant runs, M only when one
 * kernel runs per stage; each region 256-byte aligned, in this order. */
int wino_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes);

/* Eq. 3 (canonical) / eq. 4 (Legendre) for a whole layer, with a symmetric
 * cast after every bracket (Section 4.2): weight transform (skipped when
 * pretransformed), input transform, per-point channel contraction, output
 * transform, all queued on `hip_stream` (a hipStream_t, may be null = default
 * stream).  x, w_or_V, y, workspace: device pointers; d, s: host pointers.
 * Errors: EINVAL, EUNSUPPORTED, EOVERFLOW (C too large for exact fp32
 * conversion of the contraction result), EWORKSPACE, EHIP. */
int wino_conv2d(const wino_conv_desc_t* d, const void* x, const void* w_or_V, void* y,
                const wino_scales_t* s, void* workspace, size_t ws_bytes, void* hip_stream);

/* wino_conv2d for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, arithmetic and results as wino_conv2d;
 * the workspace is a device array inside the library, WINO_NOALLOC_MAX_BYTES
 * per GPU, held from the moment the library is loaded until the process ends.
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine) and never synchronises.  Its first call on a device looks up that
 * device's copy of the array (hipGetSymbolAddress, not a stream operation).
 * All calls on one GPU share the array: calls on one stream are ordered and
 * safe, calls that overlap in time on the same GPU race.
 * Errors: those of wino_conv2d; EWORKSPACE when wino_workspace_bytes(d)
 * exceeds WINO_NOALLOC_MAX_BYTES (all benchmark layers need at most 38 MiB). */
#define WINO_NOALLOC_MAX_BYTES (64u << 20)
int wino_conv2d_noalloc(const wino_conv_desc_t* d, const void* x, const void* w_or_V, void* y,
                        const wino_scales_t* s, void* hip_stream);

/* The four stages on their own (same descriptor and scales; device pointers).
 * Eq. 1 / eq. 2: w -> V. */
int wino_weight_transform(const wino_conv_desc_t* d, const void* w, void* V,
                          const wino_scales_t* s, void* hip_stream);
/* Input bracket of eq. 3 / eq. 4: x -> U. */
int wino_input_transform(const wino_conv_desc_t* d, const void* x, void* U,
                         const wino_scales_t* s, void* hip_stream);
/* Both operand transforms of a layer, x -> U and w -> V (eq. 1 / eq. 2 and the
 * input bracket of eq. 3 / eq. 4), queued as ONE kernel launch: they are
 * independent, and a layer that transforms its filters on the fly saves a
 * launch.  Results are identical to the two separate calls. */
int wino_transform_operands(const wino_conv_desc_t* d, const void* x, void* U, const void* w,
                            void* V, const wino_scales_t* s, void* hip_stream);
/* Hadamard product summed over input channels: M[p][t][k] = sum_c U V, then
 * the cast to bits_hadamard (int8 MFMA, int32 accumulation). */
int wino_contract(const wino_conv_desc_t* d, const void* U, const void* V, void* M,
                  const wino_scales_t* s, void* hip_stream);
/* Output bracket of eq. 3 / eq. 4: M -> y. */
int wino_output_transform(const wino_conv_desc_t* d, const void* M, void* y,
                          const wino_scales_t* s, void* hip_stream);
/* The Hadamard stage and the output bracket of eq. 3 / eq. 4 in ONE kernel:
 * U, V -> y with the same arithmetic and the same casts as wino_contract
 * followed by wino_output_transform (results are bit-identical), the cast
 * contraction result being kept in on-chip memory instead of a tensor M.
 * U and V in the order d->operand_layout names (FRAGMENTS is the fast one).
 * Needs bits_hadamard 8 or 9 and out_type F32 or I8 (EUNSUPPORTED otherwise). */
int wino_contract_output(const wino_conv_desc_t* d, const void* U, const void* V, void* y,
                         const wino_scales_t* s, void* hip_stream);

/* Chooses the scales of a layer on the device, from the tensors it is given
 * (dynamic quantisation; Section 4.2 casts every stage, the paper leaves the
 * choice of scales to the training framework).  On entry s->s_x and s->s_w hold
 * the scales of x and w and s->per_point selects the mode; with per_point = 1
 * the per-point arrays are filled as well: s_u_pt[p], s_v_pt[p] from the
 * maxima of point p alone, s_m from the largest point and m_shift[p] = the
 * largest shift <= WINO_MAX_M_SHIFT that does not clip point p.  On return every other field holds
 * scale = float(max |real value of that stage| / qmax), computed stage after
 * stage on the codes the previous stages produce with the scales just chosen
 * (qmax = 127, or 255 for a 9-bit Hadamard stage; 1.0 for an all-zero tensor;
 * s_y covers only positive values when relu is set).  As a side effect the
 * layer is run: V, U, M are left in the workspace and, if y is not null, the
 * output is written.  This is the one call that synchronises the stream (once
 * per cast) and it is meant to be used when a layer is set up, not per step.
 * Needs wino_calibrate_workspace_bytes() of device workspace; int8 path only;
 * C <= 1040 (the exact int32 contraction result must convert to fp32 exactly). */
int wino_calibrate_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes);
int wino_calibrate(const wino_conv_desc_t* d, const void* x, const void* w, void* y,
                   wino_scales_t* s, void* workspace, size_t ws_bytes, void* hip_stream);

/* Section 4.2, "flex" variant: the layer with TRAINED transformation matrices.
 * G_P, B_P, A_P (G, B, A when d->base is canonical) are fp32 parameters given
 * at run time; P and P^{-1} stay the fixed rational matrices.  Host arrays,
 * row-major: GP n x 3, BPT n x n (B_P transposed), APT m x n (A_P transposed);
 * entries finite, |entry| <= 2^20; they are read during the call and need not
 * outlive it. */
typedef struct {
  const float* GP;
  const float* BPT;
  const float* APT;
} wino_flex_matrices_t;

/* The stages and the layer of the flex variant.  Data flow, layouts, casts and
 * scales are those of wino_conv2d; wino_contract is shared.  The brackets with
 * P^{-1} (W1 -> V, x -> X1, M -> M1) keep their exact integer arithmetic.  A
 * bracket T q T^T with a run-time matrix T is evaluated on the integer codes q
 * in fp32, in this fixed order, every product and every sum rounded to fp32
 * and never fused:
 *     left[i][b] = ((T[i][0] q[0][b] + T[i][1] q[1][b]) + ...)
 *     out[i][j]  = ((left[i][0] T[j][0] + left[i][1] T[j][1]) + ...)
 * and is followed by the cast clamp(rint(out * float(s_prev / s_next))), the
 * exact product rounded once, ties to even; an fp32 output is
 * out * float(s_prev).  Restrictions: int8 path; Legendre base needs
 * inner_quant = 1; out_type F32 or I8; no fused variant (d->fused = ON is
 * EUNSUPPORTED, AUTO runs one kernel per stage).  Workspace of
 * wino_flex_conv2d: wino_workspace_bytes() with d->fused = OFF.
 * wino_flex_calibrate is wino_calibrate for this variant (same workspace
 * size, same rule: scale = float(max |real| / qmax) stage after stage).
 * Errors as for the static calls, plus EINVAL for a null, non-finite or
 * too large matrix entry. */
int wino_flex_weight_transform(const wino_conv_desc_t* d, const wino_flex_matrices_t* f,
                               const void* w, void* V, const wino_scales_t* s, void* hip_stream);
int wino_flex_input_transform(const wino_conv_desc_t* d, const wino_flex_matrices_t* f,
                              const void* x, void* U, const wino_scales_t* s, void* hip_stream);
int wino_flex_output_transform(const wino_conv_desc_t* d, const wino_flex_matrices_t* f,
                               const void* M, void* y, const wino_scales_t* s, void* hip_stream);
int wino_flex_conv2d(const wino_conv_desc_t* d, const wino_flex_matrices_t* f, const void* x,
                     const void* w_or_V, void* y, const wino_scales_t* s, void* workspace,
                     size_t ws_bytes, void* hip_stream);
int wino_flex_calibrate(const wino_conv_desc_t* d, const wino_flex_matrices_t* f, const void* x,
                        const void* w, void* y, wino_scales_t* s, void* workspace,
                        size_t ws_bytes, void* hip_stream);

/* Backward pass of one layer, for Winograd-aware training with fixed matrices
 * (Sections 2 and 4.2 adopt that training method; the derivative of a cast is
 * not given there and is taken as the identity, "straight-through").  Every
 * step is then the adjoint of the matching step of eq. 3, and the base change
 * of eq. 4 cancels, so d->base and d->inner_quant do not matter:
 *     dM = A dY_t A^T                      per (tile, k), A = (A^T)^T, n x m
 *     dU[p][t][c] = sum_k dM[p][t][k] * (s_v V[p][k][c])
 *     dV[p][k][c] = sum_t dM[p][t][k] * (s_u U[p][t][c])
 *     dx = sum over overlapping tiles of B dU_t B^T   (B = (B^T)^T)
 *     dw = G^T dV G
 * dy [N][H][W][K], dx [N][H][W][C], dw [K][C][3][3]: fp32 device tensors,
 * gradients with respect to the REAL output, input (s_x * code) and weights
 * (s_w * code).  U [n*n][T][C], V [n*n][K][C]: the int8 codes the forward pass
 * contracted (device).  s (host): only s_u, s_v (or, with per_point, s_u_pt,
 * s_v_pt) are read.  All arithmetic is fp32; the two contractions multiply
 * dM, cut into three bf16 pieces that together hold its upper 24 bits, by the
 * codes on the bf16 matrix instructions (exact products, fp32 accumulation:
 * fp32 accuracy; a non-finite dM gives NaN).  Sums over tiles are taken in a
 * fixed order, so results are reproducible.  Int8 path only (d->bits_in = 8).  Pixels of partial tiles
 * outside H x W receive no gradient.  d->relu, d->out_type, d->bits_hadamard
 * and d->fused are ignored: dy is the gradient at the layer's real output, a
 * ReLU or an output cast behind it is the caller's to apply to dy beforehand.
 * Inputs are only read; dx, dw and the workspace are overwritten.
 * Workspace (device, 256-byte aligned), wino_backward_workspace_bytes(): three
 * fp32 regions in this order, each rounded up to 256 bytes:
 * dM [n*n][T][K], dU [n*n][T][C], dV [n*n][K][C] (followed, for shapes with few
 * output channels and many tiles, by partial sums of dV over ranges of tiles);
 * dM, dU and dV hold those intermediate gradients when the call returns.
 * Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP. */
int wino_backward_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes);
/* *parts (host) = number of partial sums over ranges of tiles in which the dV
 * contraction of this shape is computed (a power of two, 1 ... 32); the dV
 * region of the workspace holds that many tensors.  Up to eight are added by
 * the kernel that reads dV next, more by a kernel of their own; either way
 * the first tensor holds the sum when the call returns. */
int wino_backward_dv_parts(const wino_conv_desc_t* d, int* parts);
int wino_backward(const wino_conv_desc_t* d, const void* dy, const void* U, const void* V,
                  const wino_scales_t* s, void* dx, void* dw, void* workspace, size_t ws_bytes,
                  void* hip_stream);

/* Backward pass of the flex layer (Section 4.2: G_P, B_P, A_P trained, P and
 * P^{-1} fixed; casts straight-through as in wino_backward).  Besides dx and dw,
 * now taken through the run-time matrices, it returns the gradients of the three
 * matrices.  For a bracket R = T S T^T with trained T, summed over all tiles (or
 * filters) and channels:  dT = sum dR (T S^T) + dR^T (T S),  dS = T^T dR T;
 * through a fixed bracket S1 = L S L^T:  dS = L^T dS1 L.  The inputs of the
 * trained brackets are recomputed from the forward pass's integer tensors with
 * its exact arithmetic (X1 from x, M1 from M) and dequantised (s_x1, s_m1; in the
 * canonical base x, M and s_x, s_m).
 * x [N][H][W][C], w [K][C][3][3], U, V: int8 as in the forward pass; M
 * [n*n][T][K] with the element type of d->bits_hadamard; dy, dx, dw as in
 * wino_backward; grads: device fp32 arrays, row-major, dGP n x 3, dBPT n x n,
 * dAPT m x n (gradients with respect to the entries of f->GP, f->BPT, f->APT).
 * s: the scales of the forward pass (per-tensor).  Restrictions of the flex
 * calls apply; every dimension must be positive; d->relu is ignored (mask dy
 * beforehand).  All sums are taken in a fixed order.
 * Workspace (device, 256-byte aligned), wino_flex_backward_workspace_bytes():
 * fp32 dM [n*n][T][K], dU [n*n][T][C], dV [n*n][K][C] (plus its partial sums, as
 * in wino_backward), per-tile dX [n*n][T][C] (each region rounded up to 256
 * bytes), then the partial sums of the matrix gradients.
 * Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP. */
typedef struct {
  void* dGP;
  void* dBPT;
  void* dAPT;
} wino_flex_grads_t;
int wino_flex_backward_workspace_bytes(const wino_conv_desc_t* d, size_t* bytes);
int wino_flex_backward(const wino_conv_desc_t* d, const wino_flex_matrices_t* f, const void* dy,
                       const void* x, const void* w, const void* U, const void* V, const void* M,
                       const wino_scales_t* s, void* dx, void* dw, const wino_flex_grads_t* grads,
                       void* workspace, size_t ws_bytes, void* hip_stream);

/* Measurement helper: the kernel launches wino_conv2d makes for this descriptor,
 * in order, as a comma-separated list written to the host buffer `buf`
 * (NUL-terminated; 128 bytes are always enough).  Names: weight_transform,
 * input_transform, operand_transforms (both in one launch), contraction,
 * output_transform, contraction_output, fused_layer. */
int wino_conv2d_launches(const wino_conv_desc_t* d, char* buf, size_t buf_bytes);

/* Tuning option, process-wide, for measurements and tests; the default is
 * what the library ships with.
 *   WINO_OPT_AUTO_CONOUT   1 (default): WINO_FUSED_AUTO may pick the two-kernel
 *                          form; 0: it picks between the single kernel and one
 *                          kernel per stage only
 * Errors: EINVAL (unknown option, value out of range). */
enum { WINO_OPT_AUTO_CONOUT = 1 };
int wino_set_option(int option, int value);

/* Measurement hook.  The next kernel that the calling thread launches through
 * this library records its own begin into `start_event` and its own end into
 * `stop_event` (hipEvent_t handles created by the caller, either may be null);
 * after the stream has been synchronised, hipEventElapsedTime(start, stop) is
 * that dispatch's duration without any launch or marker overhead.  The pair is
 * consumed by that one launch.  Calls queue up, oldest first, at most 8 pending
 * pairs per thread (a ninth replaces the eighth): before a call that launches
 * several kernels, k calls time its first k launches.  Always returns WINO_OK. */
int wino_profile_next_launch(void* start_event, void* stop_event);

/* Measurement helper: one register-only kernel that shows what the device
 * sustains on a unit the hot path is priced against.  WINO_PROBE_MFMA_I8:
 * every wave issues iters x 4 independent 32x32x32 int8 MFMAs;
 * WINO_PROBE_VALU_MAD24: every lane issues iters x 8 24-bit multiply-adds;
 * WINO_PROBE_MFMA_BF16: every wave issues iters x 4 independent 32x32x16
 * bf16 MFMAs (the instruction of the backward pass's contractions).
 * `blocks` work groups of 256 lanes; *work (host, may be null) receives the
 * int8 operations resp. flops (2 per multiply-accumulate) resp. lane-operations
 * of the launch; `sink` is a device int the kernel may write.  Time it with
 * wino_profile_next_launch. */
enum { WINO_PROBE_MFMA_I8 = 0, WINO_PROBE_VALU_MAD24 = 1, WINO_PROBE_MFMA_BF16 = 2 };
int wino_probe_peak(int kind, int blocks, int iters, void* sink, double* work, void* hip_stream);

/* Text of the last error on this thread ("" if none); valid until the next
 * failing call on the same thread. */
const char* wino_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* WINO_H */
