"""Backward pass of one Winograd convolution layer (Winograd-aware training, static
matrices; Sections 2 and 4.2 take that training method from prior work).

Oracle code (test infrastructure), fp64.

What is differentiated.  The layer's real-valued forward map is eq. 3,

    U = B^T X B,   V = G W G^T,   M[p] = sum_c U[p] V[p],   Y = A^T M A,

with a cast after every bracket.  The paper does not spell out the derivative of
a cast; the reading taken here is the plain straight-through estimator: a cast
passes the gradient on unchanged (for scales chosen by abs-max nothing is ever
clipped, so the clipped variant gives the same result).  With that reading

  * the gradient reaches a bracket exactly as if the bracket were unquantised, so
    each step below is the adjoint (transpose) of the corresponding linear step
    of eq. 3;
  * the base change of eq. 4 drops out: A_P^T P^{-T} = A^T etc., so the composite
    adjoints are those of the canonical matrices whatever the base of the
    forward pass;
  * the forward pass enters only through the operands of the contraction: the
    DEQUANTISED codes U = s_u * Uq and V = s_v * Vq that the forward pass really
    multiplied (per-point scales allowed).

Steps, for an incoming gradient dY [N,H,W,K] (gradient w.r.t. the real output):

  dM  = A dY_t A^T         per (tile, k); rows/columns of a partial tile that lie
                           outside the H x W output receive zero gradient
  dU[p,t,c] = sum_k dM[p,t,k] V[p,k,c]
  dV[p,k,c] = sum_t dM[p,t,k] U[p,t,c]
  dX_t = B dU B^T          per (tile, c); overlapping tiles ADD into dx, the
                           zero-padding ring is dropped
  dW  = G^T dV G           per (k, c)

Pins (tests/test_oracle_backward.py): with U and V the exact (unquantised)
transforms, dx and dw must equal the gradients of direct convolution written out
as loops; every step satisfies the adjoint identity <forward(a), b> =
<a, backward(b)> against the forward oracle; central finite differences of the
forward oracle; scalar loops for one tile of the contraction gradients.

The second half of the module is the backward pass of the flex variant (trained
G_P, B_P, A_P): gradients of the three matrices, and dx / dw through them.  Its
pins: with the static matrices it must again give the gradients of direct
convolution; central finite differences of an unquantised flex forward pass with
perturbed matrices, for entries of all three matrices and of x and w; the bracket
rule dT = dR (T S^T) + dR^T (T S) against scalar matrix products.
"""
import numpy as np

from . import matrices as mx
from .winograd import tile_counts


def _f64(T):
    return np.array([[float(v) for v in row] for row in T], dtype=np.float64)


def output_grad_tiles(dy, m):
    """dy [N,H,W,K] -> [T,m,m,K]: the adjoint of cropping the tiled output to H x W."""
    dy = np.asarray(dy, dtype=np.float64)
    N, H, W, K = dy.shape
    TH, TW = tile_counts(H, W, m)
    full = np.zeros((N, TH * m, TW * m, K))
    full[:, :H, :W, :] = dy
    out = np.zeros((N * TH * TW, m, m, K))
    t = 0
    for b in range(N):
        for ty in range(TH):
            for tx in range(TW):
                out[t] = full[b, ty * m:(ty + 1) * m, tx * m:(tx + 1) * m, :]
                t += 1
    return out


def grad_M(dy, mats):
    """dM [n*n, T, K] = A dY_t A^T, A = (A^T)^T of the canonical base."""
    AT = _f64(mats.AT)                                   # m x n
    dYt = output_grad_tiles(dy, mats.m)                  # [T,m,m,K]
    dM = np.einsum("ai,tabk,bj->ijtk", AT, dYt, AT)      # A[i,a] = AT[a,i]
    n = mats.n
    return dM.reshape(n * n, dM.shape[2], dM.shape[3])


def grad_U(dM, V):
    """dU[p,t,c] = sum_k dM[p,t,k] V[p,k,c]."""
    return np.einsum("ptk,pkc->ptc", dM, np.asarray(V, dtype=np.float64))


def grad_V(dM, U):
    """dV[p,k,c] = sum_t dM[p,t,k] U[p,t,c]."""
    return np.einsum("ptk,ptc->pkc", dM, np.asarray(U, dtype=np.float64))


def grad_x(dU, shape, mats):
    """dx [N,H,W,C]: dX_t = B dU B^T per tile, summed where tiles overlap."""
    N, H, W, C = shape
    m, r, n = mats.m, mats.r, mats.n
    pad = (r - 1) // 2
    BT = _f64(mats.BT)                                   # n x n
    T = dU.shape[1]
    dUt = dU.reshape(n, n, T, C)
    dXt = np.einsum("ia,ijtc,jb->tabc", BT, dUt, BT)     # B[a,i] = BT[i,a]
    TH, TW = tile_counts(H, W, m)
    full = np.zeros((N, TH * m + r - 1, TW * m + r - 1, C))
    t = 0
    for b in range(N):
        for ty in range(TH):
            for tx in range(TW):
                full[b, ty * m:ty * m + n, tx * m:tx * m + n, :] += dXt[t]
                t += 1
    return full[:, pad:pad + H, pad:pad + W, :]


def grad_w(dV, mats):
    """dw [K,C,r,r] = G^T dV G."""
    G = _f64(mats.G)                                     # n x r
    n = mats.n
    K, C = dV.shape[1], dV.shape[2]
    dVt = dV.reshape(n, n, K, C)
    return np.einsum("ia,ijkc,jb->kcab", G, dVt, G)


def dequantise(codes, s, s_pt=None):
    """Real operand of the contraction: codes [n*n, ., .] times its scale(s)."""
    codes = np.asarray(codes, dtype=np.float64)
    if s_pt is None:
        return codes * float(s)
    return codes * np.asarray(s_pt, dtype=np.float64)[:codes.shape[0], None, None]


def backward_layer(dy, U, V, x_shape, m, r=3):
    """All gradients of one layer.  U [n*n,T,C] and V [n*n,K,C] are the REAL
    (dequantised) operands the forward pass contracted."""
    mats = mx.Matrices(m, r, base="legendre")            # canonical G, B^T, A^T do not depend on the base
    dM = grad_M(dy, mats)
    dU = grad_U(dM, V)
    dV = grad_V(dM, U)
    return {"dM": dM, "dU": dU, "dV": dV,
            "dx": grad_x(dU, x_shape, mats), "dw": grad_w(dV, mats)}


# ---------------------------------------------------------------------------
# Flex variant (Section 4.2): G_P, B_P, A_P are trained, P and P^{-1} stay fixed.
# Forward map of one layer, casts read as identities (straight-through):
#     W1 = G_P w G_P^T         V = P^{-1} W1 P^{-T}
#     X1 = P^{-T} X P^{-1}     U = B_P^T X1 B_P
#     M[p] = sum_c U[p] V[p]   M1 = P^{-T} M P^{-1}     Y = A_P^T M1 A_P
# (canonical base: the P factors are identities and the matrices are G, B^T, A^T).
# The gradient of a bracket  R = T S T^T  with respect to T is
#     dT = dR (T S^T) + dR^T (T S),
# summed over every tile (or filter) and channel that uses T; with respect to S
# it is T^T dR T.  The forward pass enters through the REAL (dequantised) values
# it produced: w, X1 and M1 as inputs of the trained brackets, U and V as
# operands of the contraction.
# ---------------------------------------------------------------------------
def _bracket_grads(Tm, S, dR):
    """S [t, cols, cols, ch], dR [t, rows, rows, ch] -> (dT [rows, cols], dS like S)."""
    TS = np.einsum("ia,tabc->tibc", Tm, S)                       # T S
    TSt = np.einsum("ia,tbac->tibc", Tm, S)                      # T S^T
    dT = (np.einsum("tijc,tjbc->ib", dR, TSt) +
          np.einsum("tjic,tjbc->ib", dR, TS))
    dS = np.einsum("ia,tijc,jb->tabc", Tm, dR, Tm)
    return dT, dS


def flex_backward(dy, w_real, X1, M1, U, V, fm, x_shape, m, base="legendre", r=3):
    """Gradients of one flex layer.

    dy [N,H,W,K]; w_real [K,C,r,r]; X1 [T,n,n,C] and M1 [T,n,n,K]: the real
    inputs of the B_P and A_P brackets (the tiles of x resp. M itself in the
    canonical base); U [n*n,T,C], V [n*n,K,C]: the real operands of the
    contraction; fm: the matrices GP [n,r], BPT [n,n], APT [m,n]."""
    N, H, W, C = x_shape
    mats = mx.Matrices(m, r, base="legendre")
    n = mats.n
    GP, BPT, APT = (np.asarray(a, dtype=np.float64) for a in (fm.GP, fm.BPT, fm.APT))
    if base == "legendre":
        L, Pinv = _f64(mats.PinvT), _f64(mats.Pinv)            # X1 = L X L^T, V = Pinv W1 Pinv^T
    else:
        L = Pinv = np.eye(n)
    T, K = M1.shape[0], M1.shape[3]
    dYt = output_grad_tiles(dy, m)                               # [T,m,m,K]
    dAPT, dM1 = _bracket_grads(APT, np.asarray(M1, dtype=np.float64), dYt)
    dMt = np.einsum("ia,tijk,jb->tabk", L, dM1, L)               # L^T dM1 L
    dM = dMt.transpose(1, 2, 0, 3).reshape(n * n, T, K)
    dU = grad_U(dM, V)
    dV = grad_V(dM, U)
    dUt = dU.reshape(n, n, T, C).transpose(2, 0, 1, 3)           # [T,n,n,C]
    dBPT, dX1 = _bracket_grads(BPT, np.asarray(X1, dtype=np.float64), dUt)
    dXt = np.einsum("ia,tijc,jb->tabc", L, dX1, L)               # L^T dX1 L
    pad = (r - 1) // 2
    TH, TW = tile_counts(H, W, m)
    full = np.zeros((N, TH * m + r - 1, TW * m + r - 1, C))
    t = 0
    for b in range(N):
        for ty in range(TH):
            for tx in range(TW):
                full[b, ty * m:ty * m + n, tx * m:tx * m + n, :] += dXt[t]
                t += 1
    dx = full[:, pad:pad + H, pad:pad + W, :]
    dVt = dV.reshape(n, n, K, C).transpose(2, 0, 1, 3)           # [K,n,n,C]
    dW1 = np.einsum("ia,kijc,jb->kabc", Pinv, dVt, Pinv)         # Pinv^T dV Pinv
    wt = np.asarray(w_real, dtype=np.float64).transpose(0, 2, 3, 1)   # [K,r,r,C]
    dGP, dwt = _bracket_grads(GP, wt, dW1)
    return {"dAPT": dAPT, "dBPT": dBPT, "dGP": dGP, "dM": dM, "dU": dU, "dV": dV,
            "dx": dx, "dw": dwt.transpose(0, 3, 1, 2)}
