"""Quantised Winograd convolution layer, stage by stage (canonical and Legendre).

Oracle code (test infrastructure).  It follows the data flow of eq. 3 / eq. 4
with a symmetric per-tensor cast on both sides of every transformation
(Section 4.2): a cast sits after every bracket of eq. 4, i.e. on

    x, w                                   (inputs of the layer)
    X1 = P^{-T} X P^{-1},  W1 = G_P W G_P^T        (inner brackets, Legendre only)
    U  = B_P^T X1 B_P,     V  = P^{-1} W1 P^{-T}   (Winograd-domain operands)
    M  = sum_c U .* V                              (8 bit, or 9 bit, or none)
    M1 = P^{-T} M P^{-1}                           (inner bracket, Legendre only)
    y  = A_P^T M1 A_P                              (fp dequantised, or 8 bit)

(the canonical base has U = B^T X B, V = G W G^T, y = A^T M A and no inner
brackets).  The "Hadamard product" is taken after the sum over input channels:
the contraction result is what is kept on 8 or 9 bits (abstract; Section 5).

Arithmetic of one cast (this repository's reading, the paper does not fix it):
the stage matrix is T = diag(1/rho) N with integer N; the numerators
num = N Xq N^T are exact integers; the stored code is

    q_ij = clamp( rint( float32(num_ij) * mult_ij ), -qmax, +qmax ),
    mult_ij = float32( s_prev / ( (rho_i*rho_j) * s_next ) )     (double inside)

where the product of the two fp32 numbers is taken EXACTLY (it has at most 48
significant bits, so float64 holds it) and rint rounds that exact product to
the nearest integer, ties to even: one rounding for the int->float32
conversion (to nearest even), one for the cast.  qmax = 2^(bits-1) - 1.  A
stored code q stands for the real q*s.  The operands are deliberately the
kernel's fp32 values: where floating point decides an integer both sides must
take the decision from the same numbers (a fused multiply-add onto 1.5 * 2^23
computes exactly this on the GPU).

Layouts: x [N,H,W,C], w [K,C,r,r], U [n*n, T, C], V [n*n, K, C],
M [n*n, T, K], y [N,H,W,K]; Winograd point p = i*n + j.
"""
from dataclasses import dataclass, field

import numpy as np

from . import matrices as mx
from .winograd import extract_tiles, scatter_tiles


@dataclass
class LayerConfig:
    m: int = 4
    r: int = 3
    base: str = "legendre"          # "canonical" | "legendre" | "chebyshev" | "hermite"
    bits: int = 8                    # every cast except the Hadamard one
    bits_hadamard: int = 8           # 8 | 9 | 32 (32 = contraction result kept as is)
    inner_quant: bool = True         # casts on the inner brackets of eq. 4
    out_type: str = "f32"            # "f32" | "i8" | "i32"
    relu: bool = False
    per_point: bool = False          # one scale per Winograd point for U and for V


SCALE_NAMES = ("s_x", "s_x1", "s_u", "s_w", "s_w1", "s_v", "s_m", "s_m1", "s_y")


def qmax_of(bits):
    return (1 << (bits - 1)) - 1


def quantise_real(v, bits=8):
    """Symmetric per-tensor cast of a real tensor: scale = max|v| / qmax."""
    v = np.asarray(v, dtype=np.float32)
    qmax = qmax_of(bits)
    amax = float(np.max(np.abs(v))) if v.size else 0.0
    s = np.float32(amax / qmax) if amax > 0 else np.float32(1.0)
    q = np.clip(np.rint(v / s), -qmax, qmax).astype(np.int64)
    return q, s


def _imat(T):
    N, rho = mx.int_form(T)
    return np.array(N, dtype=np.int64), [int(v) for v in rho]


def _stage_dtype(Nmat, in_max):
    """int64 when every (partial) sum of the stage provably fits, else Python ints."""
    rs = max(sum(abs(int(v)) for v in row) for row in Nmat)
    return np.int64 if in_max * rs * rs < (1 << 63) else object


def sandwich_tiles(Nmat, X, dtype=np.int64):
    """num[t,i,j,c] = sum_ab N[i,a] X[t,a,b,c] N[j,b]   (exact integers)."""
    Nm, X = Nmat.astype(dtype), X.astype(dtype)
    left = np.tensordot(Nm, X, axes=([1], [1]))             # [i,t,b,c]
    both = np.tensordot(left, Nm, axes=([2], [1]))          # [i,t,c,j]
    return both.transpose(1, 0, 3, 2)


def sandwich_filters(Nmat, Wt, dtype=np.int64):
    """num[k,c,i,j] = sum_ab N[i,a] W[k,c,a,b] N[j,b]   (exact integers)."""
    Nm, Wt = Nmat.astype(dtype), Wt.astype(dtype)
    left = np.tensordot(Nm, Wt, axes=([1], [2]))            # [i,k,c,b]
    both = np.tensordot(left, Nm, axes=([3], [1]))          # [i,k,c,j]
    return both.transpose(1, 2, 0, 3)


def _int_to_f32(v):
    """Round-to-nearest-even conversion of an arbitrary Python int to float32."""
    a = abs(v)
    bl = a.bit_length()
    if bl > 24:
        sh = bl - 24
        qv, rem, half = a >> sh, a & ((1 << sh) - 1), 1 << (sh - 1)
        if rem > half or (rem == half and (qv & 1)):
            qv += 1
        a = qv << sh
    return np.float32(-float(a) if v < 0 else float(a))


def to_f32(num):
    """Integer array -> float32, one rounding (RNE), also for Python-int arrays."""
    if num.dtype != object:
        return num.astype(np.float32)
    return np.vectorize(_int_to_f32, otypes=[np.float32])(num)


def mult_table(rho_i, rho_j, s_prev, s_next):
    """float32 multipliers of one cast; s_prev may be a double (product of scales);
    s_next is one scale or an array [i, j] of per-point scales."""
    tab = np.zeros((len(rho_i), len(rho_j)), dtype=np.float32)
    per_point = np.ndim(s_next) == 2
    for i, ri in enumerate(rho_i):
        for j, rj in enumerate(rho_j):
            sn = float(s_next[i][j]) if per_point else float(s_next)
            tab[i, j] = np.float32(float(s_prev) / (float(ri * rj) * sn))
    return tab


def requant(num, mult, qmax, ij_axes):
    """clamp(rint(float32(num) * mult_ij)) with mult broadcast on ``ij_axes``."""
    shape = [1] * num.ndim
    shape[ij_axes[0]] = mult.shape[0]
    shape[ij_axes[1]] = mult.shape[1]
    prod = to_f32(num).astype(np.float64) * mult.reshape(shape).astype(np.float32).astype(np.float64)
    return np.clip(np.rint(prod), -qmax, qmax).astype(np.int64)    # exact product, one rounding


def calibrate(num, rho_i, rho_j, s_prev, qmax, ij_axes):
    """scale = float32( max |real| / qmax ), real = float64(num)*s_prev/(rho_i rho_j)."""
    shape = [1] * num.ndim
    shape[ij_axes[0]] = len(rho_i)
    shape[ij_axes[1]] = len(rho_j)
    rr = np.array([[float(a * b) for b in rho_j] for a in rho_i]).reshape(shape)
    real = (num.astype(np.float64) * float(s_prev)) / rr     # object ints: float() is RNE
    amax = float(np.max(np.abs(real))) if real.size else 0.0
    return np.float32(amax / qmax) if amax > 0 else np.float32(1.0)


def calibrate_points(num, rho_i, rho_j, s_prev, qmax, ij_axes):
    """Per-point variant of calibrate: scale[i, j] = float32(max |real[.., i, j, ..]| / qmax)."""
    out = np.ones((len(rho_i), len(rho_j)), dtype=np.float32)
    for i, ri in enumerate(rho_i):
        for j, rj in enumerate(rho_j):
            sl = [slice(None)] * num.ndim
            sl[ij_axes[0]], sl[ij_axes[1]] = i, j
            part = num[tuple(sl)]
            real = (part.astype(np.float64) * float(s_prev)) / float(ri * rj)
            amax = float(np.max(np.abs(real))) if real.size else 0.0
            if amax > 0:
                out[i, j] = np.float32(amax / qmax)
    return out


class StageMatrices:
    """Integer forms of the stage matrices one configuration uses."""

    def __init__(self, cfg):
        # the canonical matrices G, B^T, A^T do not depend on the base, so any will do there
        mats = mx.Matrices(cfg.m, cfg.r, base="legendre" if cfg.base == "canonical" else cfg.base)
        self.mats = mats
        legendre = cfg.base != "canonical"      # a polynomial base: two brackets per stage
        if legendre and cfg.inner_quant:
            self.in_inner = _imat(mats.PinvT)      # P^{-T} X P^{-1}
            self.in_outer = _imat(mats.BPT)        # B_P^T . B_P
            self.w_inner = _imat(mats.GP)          # G_P W G_P^T
            self.w_outer = _imat(mats.Pinv)        # P^{-1} . P^{-T}
            self.out_inner = _imat(mats.PinvT)     # P^{-T} M P^{-1}
            self.out_outer = _imat(mats.APT)       # A_P^T . A_P
        elif legendre:
            # Without inner casts the brackets of eq. 4 collapse: each pair of
            # factors is multiplied out ahead of time, in exact rationals.
            self.in_inner = self.w_inner = self.out_inner = None
            self.in_outer = _imat(mx.matmul(mats.BPT, mats.PinvT))
            self.w_outer = _imat(mx.matmul(mats.Pinv, mats.GP))
            self.out_outer = _imat(mx.matmul(mats.APT, mats.PinvT))
        else:
            self.in_inner = self.w_inner = self.out_inner = None
            self.in_outer = _imat(mats.BT)
            self.w_outer = _imat(mats.G)
            self.out_outer = _imat(mats.AT)


def weight_transform(wq, s_w, cfg, sm, scales, out):
    """w [K,C,r,r] int -> V [n*n, K, C]; fills s_w1 / s_v when absent."""
    qmax = qmax_of(cfg.bits)
    K, C = wq.shape[:2]
    n = cfg.m + cfg.r - 1
    cur, s_cur = wq.astype(np.int64), s_w
    if sm.w_inner is not None:
        Nm, rho = sm.w_inner
        num = sandwich_filters(Nm, cur, _stage_dtype(Nm, qmax))
        if "s_w1" not in scales:
            scales["s_w1"] = calibrate(num, rho, rho, s_cur, qmax, (2, 3))
        cur = requant(num, mult_table(rho, rho, s_cur, scales["s_w1"]), qmax, (2, 3))
        s_cur = scales["s_w1"]
        out["W1"] = cur
    Nm, rho = sm.w_outer
    num = sandwich_filters(Nm, cur, _stage_dtype(Nm, qmax))
    if "s_v" not in scales:
        cal = calibrate_points if cfg.per_point else calibrate
        scales["s_v"] = cal(num, rho, rho, s_cur, qmax, (2, 3))
    Vkc = requant(num, mult_table(rho, rho, s_cur, scales["s_v"]), qmax, (2, 3))
    out["V"] = np.ascontiguousarray(Vkc.transpose(2, 3, 0, 1).reshape(n * n, K, C))
    return out["V"]


def input_transform(xq, s_x, cfg, sm, scales, out):
    """x [N,H,W,C] int -> U [n*n, T, C]; fills s_x1 / s_u when absent."""
    qmax = qmax_of(cfg.bits)
    n = cfg.m + cfg.r - 1
    cur, s_cur = extract_tiles(xq.astype(np.int64), cfg.m, cfg.r), s_x   # [T,n,n,C]
    T, C = cur.shape[0], cur.shape[3]
    if sm.in_inner is not None:
        Nm, rho = sm.in_inner
        num = sandwich_tiles(Nm, cur, _stage_dtype(Nm, qmax))
        if "s_x1" not in scales:
            scales["s_x1"] = calibrate(num, rho, rho, s_cur, qmax, (1, 2))
        cur = requant(num, mult_table(rho, rho, s_cur, scales["s_x1"]), qmax, (1, 2))
        s_cur = scales["s_x1"]
        out["X1"] = cur
    Nm, rho = sm.in_outer
    num = sandwich_tiles(Nm, cur, _stage_dtype(Nm, qmax))
    if "s_u" not in scales:
        cal = calibrate_points if cfg.per_point else calibrate
        scales["s_u"] = cal(num, rho, rho, s_cur, qmax, (1, 2))
    Ut = requant(num, mult_table(rho, rho, s_cur, scales["s_u"]), qmax, (1, 2))
    out["U"] = np.ascontiguousarray(Ut.transpose(1, 2, 0, 3).reshape(n * n, T, C))
    return out["U"]


MAX_M_SHIFT = 8


def contraction(U, V, cfg, scales, out):
    """M[p,t,k] = sum_c U[p,t,c] V[p,k,c] (int64), then the Hadamard-stage cast.

    Per-point mode: U[p], V[p] carry their own scales, so the result of point p
    stands for M * s_u[p] * s_v[p].  Its codes get the scale s_m / 2^shift[p]:
    s_m covers the largest point, and a point whose values are smaller by a
    factor 2^s keeps s more bits, s = shift[p] <= MAX_M_SHIFT being the largest
    power of two that does not clip it.  Powers of two keep the next bracket in
    exact integers: it is fed with codes << (smax - shift[p]) at the common
    scale s_m / 2^smax, smax = max_p shift[p].
    Returns (what the output bracket is fed with, the scale of those integers)."""
    M = np.matmul(U, V.transpose(0, 2, 1))
    out["M_acc"] = M
    if not cfg.per_point:
        s_uv = float(scales["s_u"]) * float(scales["s_v"])
        if cfg.bits_hadamard == 32:
            out["M"] = M
            return M, s_uv
        qmax = qmax_of(cfg.bits_hadamard)
        if "s_m" not in scales:
            amax = float(np.max(np.abs(M.astype(np.float64) * s_uv))) if M.size else 0.0
            scales["s_m"] = np.float32(amax / qmax) if amax > 0 else np.float32(1.0)
        mult = np.float32(s_uv / float(scales["s_m"]))
        prod = M.astype(np.float32).astype(np.float64) * np.float64(mult)   # exact product
        Mq = np.clip(np.rint(prod), -qmax, qmax).astype(np.int64)
        out["M"] = Mq
        return Mq, scales["s_m"]

    assert cfg.bits_hadamard != 32, "per-point scales need a cast of the contraction result"
    qmax = qmax_of(cfg.bits_hadamard)
    n2 = M.shape[0]
    s_uv = (np.asarray(scales["s_u"], dtype=np.float64) *
            np.asarray(scales["s_v"], dtype=np.float64)).reshape(n2)
    if "s_m" not in scales or "m_shift" not in scales:
        ideal = np.zeros(n2)                       # scale that just covers point p
        for p in range(n2):
            amax = float(np.max(np.abs(M[p]))) if M[p].size else 0.0
            ideal[p] = amax * s_uv[p] / qmax
        top = float(ideal.max()) if n2 else 0.0
        scales["s_m"] = np.float32(top) if top > 0 else np.float32(1.0)
        shift = np.zeros(n2, dtype=np.int64)
        for p in range(n2):
            while shift[p] < MAX_M_SHIFT and ideal[p] * 2.0 ** (shift[p] + 1) <= float(scales["s_m"]):
                shift[p] += 1
        scales["m_shift"] = shift
    shift = np.asarray(scales["m_shift"], dtype=np.int64)
    assert shift.min() >= 0 and shift.max() <= MAX_M_SHIFT
    Mq = np.empty_like(M)
    for p in range(n2):
        mult = np.float32(s_uv[p] * 2.0 ** int(shift[p]) / float(scales["s_m"]))
        prod = M[p].astype(np.float32).astype(np.float64) * np.float64(mult)
        Mq[p] = np.clip(np.rint(prod), -qmax, qmax).astype(np.int64)
    out["M"] = Mq
    smax = int(shift.max()) if n2 else 0
    fed = Mq * (2 ** (smax - shift)).reshape(n2, 1, 1)
    return fed, float(scales["s_m"]) / 2.0 ** smax


def output_transform(Mq, s_m, shape, cfg, sm, scales, out):
    """M [n*n, T, K] -> y [N,H,W,K] (fp64 real, int8 codes, or int numerators)."""
    N, H, W = shape
    n, m = cfg.m + cfg.r - 1, cfg.m
    T, K = Mq.shape[1], Mq.shape[2]
    qmax = qmax_of(cfg.bits)
    in_max = qmax_of(cfg.bits_hadamard) if cfg.bits_hadamard != 32 else (1 << 24)
    if cfg.per_point:
        in_max <<= MAX_M_SHIFT                                   # codes arrive shifted left
        assert cfg.out_type != "i32"
    cur = Mq.reshape(n, n, T, K).transpose(2, 0, 1, 3)          # [T,n,n,K]
    s_cur = s_m
    if sm.out_inner is not None:
        Nm, rho = sm.out_inner
        num = sandwich_tiles(Nm, cur, _stage_dtype(Nm, in_max))
        if "s_m1" not in scales:
            scales["s_m1"] = calibrate(num, rho, rho, s_cur, qmax, (1, 2))
        cur = requant(num, mult_table(rho, rho, s_cur, scales["s_m1"]), qmax, (1, 2))
        s_cur = scales["s_m1"]
        in_max = qmax
        out["M1"] = cur
    Nm, rho = sm.out_outer
    num = sandwich_tiles(Nm, cur, _stage_dtype(Nm, in_max))     # [T,m,m,K]
    out["Y_num"] = num
    if cfg.out_type == "i32":
        assert all(v == 1 for v in rho), "integer output needs an integer A^T"
        y = scatter_tiles(num, N, H, W, m)
        if cfg.relu:
            y = np.maximum(y, 0)
        out["y"] = y
        return y
    rr = np.array([[float(a * b) for b in rho] for a in rho]).reshape(1, m, m, 1)
    real = (num.astype(np.float64) * float(s_cur)) / rr
    if cfg.relu:
        real = np.maximum(real, 0.0)
    out["y_real"] = scatter_tiles(real, N, H, W, m)
    if cfg.out_type == "f32":
        out["y"] = out["y_real"]
        return out["y"]
    assert cfg.out_type == "i8"
    if "s_y" not in scales:
        amax = float(np.max(np.abs(out["y_real"]))) if real.size else 0.0
        scales["s_y"] = np.float32(amax / qmax) if amax > 0 else np.float32(1.0)
    q = requant(num, mult_table(rho, rho, s_cur, scales["s_y"]), qmax, (1, 2))
    if cfg.relu:
        q = np.maximum(q, 0)
    out["y"] = scatter_tiles(q, N, H, W, m)
    return out["y"]


def run_layer(xq, wq, s_x, s_w, cfg, scales=None):
    """The whole quantised layer.  Returns (stages dict, scales dict).

    ``scales`` missing entries are calibrated stage after stage on this very
    tensor (scale = float32(max|real| / qmax), 1.0 for an all-zero tensor);
    present entries are used unchanged.
    """
    scales = {} if scales is None else dict(scales)
    scales["s_x"], scales["s_w"] = np.float32(s_x), np.float32(s_w)
    sm = StageMatrices(cfg)
    out = {}
    xq = np.asarray(xq)
    N, H, W, _ = xq.shape
    V = weight_transform(np.asarray(wq), scales["s_w"], cfg, sm, scales, out)
    U = input_transform(xq, scales["s_x"], cfg, sm, scales, out)
    Mq, s_m = contraction(U, V, cfg, scales, out)
    output_transform(Mq, s_m, (N, H, W), cfg, sm, scales, out)
    return out, scales
