"""Unquantised Winograd convolution, canonical (eq. 3) and Legendre base (eq. 4).

Oracle code (test infrastructure).  The tiling is the usual one for stride 1,
pad 1: with n = m + r - 1, tile (ty, tx) of image b reads input rows
ty*m - 1 ... ty*m - 1 + n - 1 (zeros outside the image, and zeros beyond the
bottom/right edge when H or W is not a multiple of m) and produces output rows
ty*m ... ty*m + m - 1, cropped to H x W.  Tiles are numbered
t = (b*TH + ty)*TW + tx with TH = ceil(H/m), TW = ceil(W/m).

Eq. 4 is taken with P^{-1} as the right factor of the inner input bracket
(the printed P there would make eq. 4 differ from eq. 3; see
``tests/test_oracle_matrices.py``).
"""
import numpy as np

from . import matrices as mx


def tile_counts(H, W, m):
    return -(-H // m), -(-W // m)


def extract_tiles(x, m, r):
    """x [N,H,W,C] -> d [T, n, n, C] (same dtype), zero padded."""
    x = np.asarray(x)
    N, H, W, C = x.shape
    n = m + r - 1
    pad = (r - 1) // 2
    TH, TW = tile_counts(H, W, m)
    xp = np.zeros((N, TH * m + r - 1, TW * m + r - 1, C), dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    d = np.zeros((N * TH * TW, n, n, C), dtype=x.dtype)
    t = 0
    for b in range(N):
        for ty in range(TH):
            for tx in range(TW):
                d[t] = xp[b, ty * m:ty * m + n, tx * m:tx * m + n, :]
                t += 1
    return d


def scatter_tiles(Y, N, H, W, m):
    """Y [T, m, m, K] -> y [N,H,W,K], cropping partial tiles."""
    TH, TW = tile_counts(H, W, m)
    K = Y.shape[-1]
    full = np.zeros((N, TH * m, TW * m, K), dtype=Y.dtype)
    t = 0
    for b in range(N):
        for ty in range(TH):
            for tx in range(TW):
                full[b, ty * m:(ty + 1) * m, tx * m:(tx + 1) * m, :] = Y[t]
                t += 1
    return full[:, :H, :W, :]


def _f64(T):
    return np.array([[float(v) for v in row] for row in T], dtype=np.float64)


def conv_eq3(x, w, mats, dtype=np.float64):
    """A^T [ (G W G^T) .* (B^T X B) ] A summed over input channels (eq. 3)."""
    m, r = mats.m, mats.r
    x = np.asarray(x, dtype=dtype)
    w = np.asarray(w, dtype=dtype)
    N, H, W, C = x.shape
    G, BT, AT = _f64(mats.G), _f64(mats.BT), _f64(mats.AT)
    d = extract_tiles(x, m, r)                                # [T,n,n,C]
    U = np.einsum("ia,tabc,jb->tijc", BT, d, BT)              # B^T X B
    V = np.einsum("ia,kcab,jb->kcij", G, w, G)                # G W G^T
    M = np.einsum("tijc,kcij->tijk", U, V)                    # Hadamard + sum_c
    Y = np.einsum("ia,tabk,jb->tijk", AT, M, AT)              # A^T M A
    return scatter_tiles(Y, N, H, W, m)


def conv_eq4(x, w, mats, dtype=np.float64, literal_print=False):
    """Eq. 4: the same computation routed through the Legendre base.

    ``literal_print=True`` evaluates the input bracket exactly as printed
    (right factor P instead of P^{-1}); it exists only so that a test can show
    that the printed form is not a convolution.
    """
    m, r = mats.m, mats.r
    x = np.asarray(x, dtype=dtype)
    w = np.asarray(w, dtype=dtype)
    N, H, W, C = x.shape
    GP, BPT, APT = _f64(mats.GP), _f64(mats.BPT), _f64(mats.APT)
    PinvT, Pinv, P = _f64(mats.PinvT), _f64(mats.Pinv), _f64(mats.P)
    d = extract_tiles(x, m, r)
    # input: B_P^T ( P^{-T} X P^{-1} ) B_P
    right = P if literal_print else Pinv
    X1 = np.einsum("ia,tabc,bj->tijc", PinvT, d, right)
    U = np.einsum("ia,tabc,jb->tijc", BPT, X1, BPT)
    # weights: P^{-1} ( G_P W G_P^T ) P^{-T}
    W1 = np.einsum("ia,kcab,jb->kcij", GP, w, GP)
    V = np.einsum("ia,kcab,bj->kcij", Pinv, W1, PinvT)
    M = np.einsum("tijc,kcij->tijk", U, V)
    # output: A_P^T [ P^{-T} M P^{-1} ] A_P
    M1 = np.einsum("ia,tabk,bj->tijk", PinvT, M, Pinv)
    Y = np.einsum("ia,tabk,jb->tijk", APT, M1, APT)
    return scatter_tiles(Y, N, H, W, m)


# ---- exact-rational single tile (tiny inputs) ------------------------------

def tile_eq3_fraction(X, Wk, mats):
    """One n x n tile X and one r x r filter (lists of Fractions) -> m x m."""
    BT, G, AT = mats.BT, mats.G, mats.AT
    U = mx.matmul(mx.matmul(BT, X), mx.transpose(BT))
    V = mx.matmul(mx.matmul(G, Wk), mx.transpose(G))
    n = mats.n
    M = [[U[i][j] * V[i][j] for j in range(n)] for i in range(n)]
    return mx.matmul(mx.matmul(AT, M), mx.transpose(AT))


def tile_eq4_fraction(X, Wk, mats):
    PinvT, Pinv = mats.PinvT, mats.Pinv
    X1 = mx.matmul(mx.matmul(PinvT, X), Pinv)
    U = mx.matmul(mx.matmul(mats.BPT, X1), mx.transpose(mats.BPT))
    W1 = mx.matmul(mx.matmul(mats.GP, Wk), mx.transpose(mats.GP))
    V = mx.matmul(mx.matmul(Pinv, W1), PinvT)
    n = mats.n
    M = [[U[i][j] * V[i][j] for j in range(n)] for i in range(n)]
    M1 = mx.matmul(mx.matmul(PinvT, M), Pinv)
    return mx.matmul(mx.matmul(mats.APT, M1), mx.transpose(mats.APT))


def tile_direct_fraction(X, Wk, m, r):
    """Valid correlation of an n x n tile with an r x r filter -> m x m."""
    return [[sum(X[i + a][j + b] * Wk[a][b] for a in range(r) for b in range(r))
             for j in range(m)] for i in range(m)]
