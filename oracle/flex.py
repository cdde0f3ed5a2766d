"""Quantised Winograd layer with run-time ("flex") transformation matrices.

Oracle code (test infrastructure).  Section 4.2 runs two variants of the
quantised layer: *static*, whose matrices are the fixed rational ones, and
*flex*, in which G_P, B_P and A_P (G, B, A in the canonical base) are trained
fp32 parameters while P and P^{-1} stay fixed.  This module states the forward
pass of the flex variant for given matrices; where the matrices come from
(training) is outside of it.

Data flow and casts are those of ``quantised.py``.  The brackets with the fixed
P^{-1} factors keep their exact integer arithmetic; a bracket with a run-time
matrix T (fp32, rows x cols) is evaluated on the integer codes in fp32, in a
fixed order that both sides of a parity test can follow (this repository's
reading; the paper fixes no arithmetic):

    left[i][b] = ((T[i][0]*x[0][b] + T[i][1]*x[1][b]) + ... )        a ascending
    out[i][j]  = ((left[i][0]*T[j][0] + left[i][1]*T[j][1]) + ... )  b ascending

with every product and every sum rounded to fp32 (no fused multiply-add).  The
cast that follows is the one of ``quantised.py`` with one multiplier for the
whole tensor, ``mult = float32(s_prev / s_next)``: the exact product
``out * mult`` rounded once to the nearest integer, ties to even, clamped.
An fp32 output is ``out * float32(s_prev)`` in fp32.

Parity status: the bracket arithmetic is pinned by the cases in which fp32 is
exact (integer and dyadic matrices, where it must reproduce ``quantised.py``
bit for bit), by an fp64 evaluation of the same formula with the same
(arbitrary, non-symmetric) matrices at high bit widths, and by brute-force loops
on one tile.  Absolute outputs for trained matrices: parity unpinned (the paper
publishes no trained matrices).
"""
from dataclasses import dataclass

import numpy as np

from . import matrices as mx
from . import quantised as oq
from .winograd import extract_tiles, scatter_tiles


@dataclass
class FlexMatrices:
    """fp32 matrices of the trainable brackets: GP [n,r], BPT [n,n], APT [m,n]
    (read as G, B^T, A^T when the layer runs in the canonical base)."""
    GP: np.ndarray
    BPT: np.ndarray
    APT: np.ndarray

    @staticmethod
    def from_exact(m, r=3, base="legendre"):
        """The static matrices rounded to fp32 (the starting point of training)."""
        mats = mx.Matrices(m, r)
        pick = (mats.GP, mats.BPT, mats.APT) if base == "legendre" else (mats.G, mats.BT, mats.AT)
        return FlexMatrices(*[np.array([[float(v) for v in row] for row in T], dtype=np.float32)
                              for T in pick])


def fsandwich(Tf, X):
    """out[..., i, j, :] = T X T^T on axes (-3, -2) of X, in the fp32 order above.

    X [..., cols, cols, ch] holds integer codes; the result is float32
    [..., rows, rows, ch]."""
    Tf = np.asarray(Tf, dtype=np.float32)
    rows, cols = Tf.shape
    Xf = np.asarray(X).astype(np.float32)
    assert Xf.shape[-3] == cols and Xf.shape[-2] == cols
    left = []                                           # left[i]: [..., b, ch]
    for i in range(rows):
        acc = Tf[i, 0] * Xf[..., 0, :, :]
        for a in range(1, cols):
            acc = acc + Tf[i, a] * Xf[..., a, :, :]
        left.append(acc)
    out = np.empty(Xf.shape[:-3] + (rows, rows, Xf.shape[-1]), dtype=np.float32)
    for i in range(rows):
        for j in range(rows):
            acc = left[i][..., 0, :] * Tf[j, 0]
            for b in range(1, cols):
                acc = acc + left[i][..., b, :] * Tf[j, b]
            out[..., i, j, :] = acc
    assert out.dtype == np.float32
    return out


def fcast(val, s_prev, s_next, qmax):
    """clamp(rint(val * float32(s_prev / s_next))): exact product, one rounding."""
    mult = np.float32(float(s_prev) / float(s_next))
    prod = val.astype(np.float64) * np.float64(mult)
    return np.clip(np.rint(prod), -qmax, qmax).astype(np.int64)


def fcalibrate(val, s_prev, qmax):
    amax = float(np.max(np.abs(val.astype(np.float64)))) * float(s_prev) if val.size else 0.0
    return np.float32(amax / qmax) if amax > 0 else np.float32(1.0)


def run_layer_flex(xq, wq, s_x, s_w, cfg, fm, scales=None):
    """The flex layer.  ``cfg`` is a quantised.LayerConfig (base legendre needs
    inner_quant; out_type "f32" or "i8").  Returns (stages, scales) like
    quantised.run_layer."""
    assert cfg.out_type in ("f32", "i8")
    legendre = cfg.base == "legendre"
    assert cfg.inner_quant or not legendre, "flex Legendre layers cast the inner brackets"
    scales = {} if scales is None else dict(scales)
    scales["s_x"], scales["s_w"] = np.float32(s_x), np.float32(s_w)
    qmax = oq.qmax_of(cfg.bits)
    m, r = cfg.m, cfg.r
    n = m + r - 1
    mats = mx.Matrices(m, r)
    PinvT, Pinv = oq._imat(mats.PinvT), oq._imat(mats.Pinv)
    out = {}
    xq, wq = np.asarray(xq), np.asarray(wq)
    N, H, W, C = xq.shape
    K = wq.shape[0]

    # filters: W1 = Q(G_P w G_P^T) in fp32, V = Q(P^{-1} W1 P^{-T}) in integers
    wt = wq.astype(np.int64).transpose(0, 2, 3, 1)                     # [K,r,r,C]
    val = fsandwich(fm.GP, wt)                                          # [K,n,n,C]
    first = "s_w1" if legendre else "s_v"
    if first not in scales:
        scales[first] = fcalibrate(val, scales["s_w"], qmax)
    cur = fcast(val, scales["s_w"], scales[first], qmax)
    if legendre:
        out["W1"] = cur.transpose(0, 3, 1, 2)                          # [K,C,n,n]
        Nm, rho = Pinv
        num = oq.sandwich_filters(Nm, out["W1"], oq._stage_dtype(Nm, qmax))
        if "s_v" not in scales:
            scales["s_v"] = oq.calibrate(num, rho, rho, scales["s_w1"], qmax, (2, 3))
        Vkc = oq.requant(num, oq.mult_table(rho, rho, scales["s_w1"], scales["s_v"]), qmax, (2, 3))
    else:
        Vkc = cur.transpose(0, 3, 1, 2)
    V = np.ascontiguousarray(Vkc.transpose(2, 3, 0, 1).reshape(n * n, K, C))
    out["V"] = V

    # activations: X1 = Q(P^{-T} X P^{-1}) in integers, U = Q(B_P^T X1 B_P) in fp32
    cur = extract_tiles(xq.astype(np.int64), m, r)                      # [T,n,n,C]
    T = cur.shape[0]
    s_cur = scales["s_x"]
    if legendre:
        Nm, rho = PinvT
        num = oq.sandwich_tiles(Nm, cur, oq._stage_dtype(Nm, qmax))
        if "s_x1" not in scales:
            scales["s_x1"] = oq.calibrate(num, rho, rho, s_cur, qmax, (1, 2))
        cur = oq.requant(num, oq.mult_table(rho, rho, s_cur, scales["s_x1"]), qmax, (1, 2))
        s_cur = scales["s_x1"]
        out["X1"] = cur
    val = fsandwich(fm.BPT, cur)
    if "s_u" not in scales:
        scales["s_u"] = fcalibrate(val, s_cur, qmax)
    Ut = fcast(val, s_cur, scales["s_u"], qmax)
    U = np.ascontiguousarray(Ut.transpose(1, 2, 0, 3).reshape(n * n, T, C))
    out["U"] = U

    Mq, s_m = oq.contraction(U, V, cfg, scales, out)

    # output: M1 = Q(P^{-T} M P^{-1}) in integers, y = A_P^T M1 A_P in fp32
    in_max = oq.qmax_of(cfg.bits_hadamard) if cfg.bits_hadamard != 32 else (1 << 24)
    cur = Mq.reshape(n, n, T, K).transpose(2, 0, 1, 3)                  # [T,n,n,K]
    s_cur = s_m
    if legendre:
        Nm, rho = PinvT
        num = oq.sandwich_tiles(Nm, cur, oq._stage_dtype(Nm, in_max))
        if "s_m1" not in scales:
            scales["s_m1"] = oq.calibrate(num, rho, rho, s_cur, qmax, (1, 2))
        cur = oq.requant(num, oq.mult_table(rho, rho, s_cur, scales["s_m1"]), qmax, (1, 2))
        s_cur = scales["s_m1"]
        out["M1"] = cur
    val = fsandwich(fm.APT, cur)                                        # [T,m,m,K]
    out["Y_val"] = val
    real = val * np.float32(float(s_cur))                               # fp32 product
    if cfg.relu:
        real = np.maximum(real, np.float32(0))
    out["y_real"] = scatter_tiles(real, N, H, W, m)
    if cfg.out_type == "f32":
        out["y"] = out["y_real"]
        return out, scales
    if "s_y" not in scales:
        crop = scatter_tiles(np.maximum(val, np.float32(0)) if cfg.relu else val, N, H, W, m)
        scales["s_y"] = fcalibrate(crop, s_cur, qmax)
    q = fcast(val, s_cur, scales["s_y"], qmax)
    if cfg.relu:
        q = np.maximum(q, 0)
    out["y"] = scatter_tiles(q, N, H, W, m)
    return out, scales
