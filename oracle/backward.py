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
