"""Direct 2-D convolution (cross-correlation, stride 1, zero pad 1): the definition.

Oracle code (test infrastructure).  y[n,h,w,k] = sum_{c,a,b} x[n,h+a-1,w+b-1,c]
* w[k,c,a,b] with zeros outside the image -- the O(k^2)-multiplications-per-
output baseline of Section 1.  Activations are NHWC, weights KCRS.
"""
from fractions import Fraction

import numpy as np


def direct_conv_loops(x, w, zero=0):
    """Seven nested loops; any element type supporting + and * (tiny inputs)."""
    N, H, W, C = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    K, r = len(w), len(w[0][0])
    pad = (r - 1) // 2
    y = [[[[zero for _ in range(K)] for _ in range(W)] for _ in range(H)]
         for _ in range(N)]
    for n in range(N):
        for h in range(H):
            for ww in range(W):
                for k in range(K):
                    acc = zero
                    for c in range(C):
                        for a in range(r):
                            for b in range(r):
                                hh, wb = h + a - pad, ww + b - pad
                                if 0 <= hh < H and 0 <= wb < W:
                                    acc = acc + x[n][hh][wb][c] * w[k][c][a][b]
                    y[n][h][ww][k] = acc
    return y


def direct_conv(x, w, dtype=np.float64):
    """Vectorised over (n, h, w, k): sum of r*r shifted channel contractions.

    ``dtype`` float64 for real inputs, int64 for integer inputs (exact).
    """
    x = np.asarray(x).astype(dtype)
    w = np.asarray(w).astype(dtype)
    N, H, W, C = x.shape
    K, C2, r, r2 = w.shape
    assert C == C2 and r == r2
    pad = (r - 1) // 2
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    y = np.zeros((N, H, W, K), dtype=dtype)
    for a in range(r):
        for b in range(r):
            y += np.matmul(xp[:, a:a + H, b:b + W, :], w[:, :, a, b].T)
    return y


def to_fraction_nested(arr):
    arr = np.asarray(arr)
    if arr.ndim == 0:
        return Fraction(int(arr))
    return [to_fraction_nested(a) for a in arr]
