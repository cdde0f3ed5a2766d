"""Pins of the backward-pass oracle (CPU only).

The gradients of direct convolution, written out below from its definition
y[n,h,w,k] = sum x[n,h+a-1,w+b-1,c] w[k,c,a,b], are the independent reference:
with unquantised operands the Winograd backward pass must reproduce them.
"""
import numpy as np
import pytest

from oracle import backward as bw
from oracle import matrices as mx
from oracle import winograd as wg


def direct_grads(x, w, dy):
    """dx and dw of zero-padded stride-1 cross-correlation, by shifted slices."""
    N, H, W, C = x.shape
    K = w.shape[0]
    xp = np.zeros((N, H + 2, W + 2, C))
    xp[:, 1:H + 1, 1:W + 1, :] = x
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    for a in range(3):
        for b in range(3):
            # y[:, h, w, k] += xp[:, h + a, w + b, c] * w[k, c, a, b]
            dw[:, :, a, b] = np.einsum("nhwc,nhwk->kc", xp[:, a:a + H, b:b + W, :], dy)
            dxp[:, a:a + H, b:b + W, :] += np.einsum("nhwk,kc->nhwc", dy, w[:, :, a, b])
    return dxp[:, 1:H + 1, 1:W + 1, :], dw


def exact_operands(x, w, mats):
    G, BT = bw._f64(mats.G), bw._f64(mats.BT)
    n = mats.n
    d = wg.extract_tiles(x, mats.m, mats.r)                         # [T,n,n,C]
    U = np.einsum("ia,tabc,jb->ijtc", BT, d, BT).reshape(n * n, d.shape[0], x.shape[3])
    V = np.einsum("ia,kcab,jb->ijkc", G, w, G).reshape(n * n, w.shape[0], w.shape[1])
    return U, V


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("shape", [(2, 8, 8, 3, 2), (1, 7, 9, 2, 3), (2, 5, 13, 1, 2)])
def test_unquantised_backward_equals_direct_gradients(m, shape):
    N, H, W, C, K = shape
    rng = np.random.default_rng(100 * m + H)
    x = rng.standard_normal((N, H, W, C))
    w = rng.standard_normal((K, C, 3, 3))
    dy = rng.standard_normal((N, H, W, K))
    mats = mx.Matrices(m, 3)
    U, V = exact_operands(x, w, mats)
    got = bw.backward_layer(dy, U, V, x.shape, m)
    dx, dw = direct_grads(x, w, dy)
    scale = 10.0 ** {2: 0, 4: 1, 6: 3}[m]          # conditioning of the F(m,3) matrices in fp64
    assert np.abs(got["dx"] - dx).max() <= 1e-12 * scale * np.abs(dx).max()
    assert np.abs(got["dw"] - dw).max() <= 1e-12 * scale * np.abs(dw).max()


@pytest.mark.parametrize("m", [2, 4, 6])
def test_each_step_is_the_adjoint_of_its_forward_step(m):
    rng = np.random.default_rng(7 + m)
    mats = mx.Matrices(m, 3)
    n = mats.n
    N, H, W, C, K = 2, 9, 6, 3, 2
    TH, TW = wg.tile_counts(H, W, m)
    T = N * TH * TW
    AT, BT, G = bw._f64(mats.AT), bw._f64(mats.BT), bw._f64(mats.G)
    # output bracket + crop
    M = rng.standard_normal((n * n, T, K))
    dy = rng.standard_normal((N, H, W, K))
    Y = np.einsum("ia,abtk,jb->tijk", AT, M.reshape(n, n, T, K), AT)
    y = wg.scatter_tiles(Y, N, H, W, m)
    assert np.isclose((y * dy).sum(), (M * bw.grad_M(dy, mats)).sum(), rtol=1e-11)
    # tiling + input bracket
    x = rng.standard_normal((N, H, W, C))
    dU = rng.standard_normal((n * n, T, C))
    d = wg.extract_tiles(x, m, 3)
    U = np.einsum("ia,tabc,jb->ijtc", BT, d, BT).reshape(n * n, T, C)
    assert np.isclose((U * dU).sum(), (x * bw.grad_x(dU, x.shape, mats)).sum(), rtol=1e-11)
    # filter bracket
    w = rng.standard_normal((K, C, 3, 3))
    dV = rng.standard_normal((n * n, K, C))
    V = np.einsum("ia,kcab,jb->ijkc", G, w, G).reshape(n * n, K, C)
    assert np.isclose((V * dV).sum(), (w * bw.grad_w(dV, mats)).sum(), rtol=1e-11)


def test_finite_differences_of_the_forward_oracle():
    m = 4
    rng = np.random.default_rng(11)
    mats = mx.Matrices(m, 3)
    x = rng.standard_normal((1, 6, 7, 2))
    w = rng.standard_normal((3, 2, 3, 3))
    dy = rng.standard_normal((1, 6, 7, 3))
    U, V = exact_operands(x, w, mats)
    g = bw.backward_layer(dy, U, V, x.shape, m)
    loss = lambda xx, ww: float((wg.conv_eq3(xx, ww, mats) * dy).sum())
    h = 1e-3                                       # the loss is bilinear: central differences are exact
    for idx in [(0, 0, 0, 0), (0, 5, 6, 1), (0, 3, 2, 1)]:
        e = np.zeros_like(x); e[idx] = h
        assert np.isclose((loss(x + e, w) - loss(x - e, w)) / (2 * h), g["dx"][idx], rtol=1e-8, atol=1e-9)
    for idx in [(0, 0, 0, 0), (2, 1, 2, 2), (1, 0, 1, 2)]:
        e = np.zeros_like(w); e[idx] = h
        assert np.isclose((loss(x, w + e) - loss(x, w - e)) / (2 * h), g["dw"][idx], rtol=1e-8, atol=1e-9)


def test_contraction_gradients_by_scalar_loops_on_quantised_operands():
    rng = np.random.default_rng(3)
    n2, T, C, K = 16, 3, 2, 4
    Uq = rng.integers(-127, 128, (n2, T, C))
    Vq = rng.integers(-127, 128, (n2, K, C))
    s_u_pt = rng.uniform(0.01, 0.1, n2)
    s_v = 0.03
    U = bw.dequantise(Uq, None, s_u_pt)
    V = bw.dequantise(Vq, s_v)
    dM = rng.standard_normal((n2, T, K))
    dU, dV = bw.grad_U(dM, V), bw.grad_V(dM, U)
    for p in range(n2):
        for c in range(C):
            for t in range(T):
                ref = sum(dM[p, t, k] * (s_v * Vq[p, k, c]) for k in range(K))
                assert abs(dU[p, t, c] - ref) < 1e-12 * max(1.0, abs(ref))
            for k in range(K):
                ref = sum(dM[p, t, k] * (s_u_pt[p] * Uq[p, t, c]) for t in range(T))
                assert abs(dV[p, k, c] - ref) < 1e-12 * max(1.0, abs(ref))


def test_gradient_outside_the_cropped_output_is_dropped():
    # H = 5 with m = 4: the second tile row owns output rows 4..7, of which only
    # row 4 exists.  Changing nothing but the tile padding must not change dM.
    mats = mx.Matrices(4, 3)
    rng = np.random.default_rng(5)
    dy = rng.standard_normal((1, 5, 4, 1))
    t = bw.output_grad_tiles(dy, 4)
    assert t.shape == (2, 4, 4, 1)
    assert np.array_equal(t[1, 0], dy[0, 4]) and not t[1, 1:].any()


# ---------------------------------------------------------------------------
# flex variant: gradients of the trained matrices
# ---------------------------------------------------------------------------
def flex_forward_real(x, w, GP, BPT, APT, mats, base):
    """Unquantised flex layer (casts as identities), plus the tensors the backward pass needs."""
    n, m = mats.n, mats.m
    L = bw._f64(mats.PinvT) if base == "legendre" else np.eye(n)
    Pinv = bw._f64(mats.Pinv) if base == "legendre" else np.eye(n)
    d = wg.extract_tiles(x, m, 3)                                        # [T,n,n,C]
    X1 = np.einsum("ia,tabc,jb->tijc", L, d, L)
    Ut = np.einsum("ia,tabc,jb->tijc", BPT, X1, BPT)
    W1 = np.einsum("ia,kcab,jb->kijc", GP, w, GP)                         # [K,n,n,C]
    Vt = np.einsum("ia,kabc,jb->kijc", Pinv, W1, Pinv)
    M = np.einsum("tijc,kijc->tijk", Ut, Vt)
    M1 = np.einsum("ia,tabk,jb->tijk", L, M, L)
    Y = np.einsum("ia,tabk,jb->tijk", APT, M1, APT)
    N, H, W, _ = x.shape
    T, C, K = d.shape[0], x.shape[3], w.shape[0]
    U = Ut.transpose(1, 2, 0, 3).reshape(n * n, T, C)
    V = Vt.transpose(1, 2, 0, 3).reshape(n * n, K, C)
    return wg.scatter_tiles(Y, N, H, W, m), X1, M1, U, V


def flex_case(m, base, seed, perturb):
    from oracle.flex import FlexMatrices
    rng = np.random.default_rng(seed)
    mats = mx.Matrices(m, 3)
    fm = FlexMatrices.from_exact(m, 3, base)
    GP, BPT, APT = (np.asarray(a, dtype=np.float64) for a in (fm.GP, fm.BPT, fm.APT))
    if perturb:                                   # "trained" matrices: no longer a convolution
        GP = GP + 0.05 * rng.standard_normal(GP.shape)
        BPT = BPT + 0.05 * rng.standard_normal(BPT.shape)
        APT = APT + 0.05 * rng.standard_normal(APT.shape)
    x = rng.standard_normal((2, 7, 6, 2))
    w = rng.standard_normal((3, 2, 3, 3))
    dy = rng.standard_normal((2, 7, 6, 3))
    return mats, FlexMatrices(GP, BPT, APT), x, w, dy


@pytest.mark.parametrize("m,base", [(2, "legendre"), (4, "legendre"), (4, "canonical"), (6, "legendre")])
def test_flex_backward_with_static_matrices_equals_the_static_backward(m, base):
    mats, fm, x, w, dy = flex_case(m, base, 21 + m, perturb=False)
    # exact static matrices in fp64 (from_exact rounds to fp32, which would blur the comparison)
    pick = (mats.GP, mats.BPT, mats.APT) if base == "legendre" else (mats.G, mats.BT, mats.AT)
    fm.GP, fm.BPT, fm.APT = (bw._f64(a) for a in pick)
    y, X1, M1, U, V = flex_forward_real(x, w, fm.GP, fm.BPT, fm.APT, mats, base)
    assert np.allclose(y, wg.conv_eq3(x, w, mats), rtol=0, atol=1e-7 * 10.0 ** m)
    got = bw.flex_backward(dy, w, X1, M1, U, V, fm, x.shape, m, base)
    dx, dw = direct_grads(x, w, dy)
    scale = 10.0 ** {2: 1, 4: 3, 6: 6}[m]          # conditioning of the Legendre brackets in fp64
    assert np.abs(got["dx"] - dx).max() <= 1e-12 * scale * np.abs(dx).max()
    assert np.abs(got["dw"] - dw).max() <= 1e-12 * scale * np.abs(dw).max()


@pytest.mark.parametrize("m,base", [(2, "legendre"), (4, "legendre"), (4, "canonical")])
def test_flex_matrix_gradients_by_finite_differences(m, base):
    mats, fm, x, w, dy = flex_case(m, base, 5 + m, perturb=True)
    y, X1, M1, U, V = flex_forward_real(x, w, fm.GP, fm.BPT, fm.APT, mats, base)
    g = bw.flex_backward(dy, w, X1, M1, U, V, fm, x.shape, m, base)

    def loss(GP, BPT, APT, xx=x, ww=w):
        return float((flex_forward_real(xx, ww, GP, BPT, APT, mats, base)[0] * dy).sum())
    h = 1e-5
    rng = np.random.default_rng(0)
    for name in ("GP", "BPT", "APT"):
        Tm = getattr(fm, name)
        for _ in range(4):
            i, j = rng.integers(Tm.shape[0]), rng.integers(Tm.shape[1])
            args = {k: getattr(fm, k).copy() for k in ("GP", "BPT", "APT")}
            args[name][i, j] += h
            up = loss(**args)
            args[name][i, j] -= 2 * h
            dn = loss(**args)
            fd = (up - dn) / (2 * h)               # the loss is quadratic in each matrix: O(h^2) error
            ref = g["d" + name][i, j]
            assert abs(fd - ref) <= 1e-6 * max(1.0, abs(ref)), (name, i, j, fd, ref)
    # and the data gradients with perturbed matrices (the layer is still bilinear in x and w)
    e = np.zeros_like(x); e[1, 3, 2, 1] = 1e-3
    fd = (loss(fm.GP, fm.BPT, fm.APT, xx=x + e) - loss(fm.GP, fm.BPT, fm.APT, xx=x - e)) / 2e-3
    assert np.isclose(fd, g["dx"][1, 3, 2, 1], rtol=1e-8, atol=1e-8)
    e = np.zeros_like(w); e[2, 1, 0, 2] = 1e-3
    fd = (loss(fm.GP, fm.BPT, fm.APT, ww=w + e) - loss(fm.GP, fm.BPT, fm.APT, ww=w - e)) / 2e-3
    assert np.isclose(fd, g["dw"][2, 1, 0, 2], rtol=1e-8, atol=1e-8)


def test_bracket_gradient_by_scalar_loops():
    rng = np.random.default_rng(9)
    Tm = rng.standard_normal((2, 3))
    S = rng.standard_normal((4, 3, 3, 2))          # [tile, a, b, ch]
    dR = rng.standard_normal((4, 2, 2, 2))
    dT, dS = bw._bracket_grads(Tm, S, dR)
    ref = np.zeros_like(Tm)
    for t in range(4):
        for c in range(2):
            s, g = S[t, :, :, c], dR[t, :, :, c]
            ref += g @ (Tm @ s.T) + g.T @ (Tm @ s)
            assert np.allclose(dS[t, :, :, c], Tm.T @ g @ Tm)
    assert np.allclose(dT, ref)


def test_straight_through_gradients_reduce_the_error_of_a_quantised_flex_layer():
    """The reading of the cast derivative is only useful if descending along the gradients it
    gives improves the QUANTISED layer.  Starting from perturbed matrices, a few normalised
    gradient steps on G_P, B_P, A_P (scales re-calibrated each step, 9-bit Hadamard stage)
    must bring the output closer to direct convolution of the same dequantised inputs."""
    from helpers import small_layer
    from oracle import direct, flex, quantised as q
    m, base = 4, "legendre"
    N, H, W, C, K = 2, 8, 8, 16, 16
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=5)
    y_ref = direct.direct_conv(xq.astype(np.float64) * float(s_x), wq.astype(np.float64) * float(s_w))
    rng = np.random.default_rng(0)
    fm = flex.FlexMatrices.from_exact(m, base=base)
    for name in ("GP", "BPT", "APT"):
        a = getattr(fm, name)
        setattr(fm, name, (a + 0.03 * rng.standard_normal(a.shape) * np.abs(a).max()).astype(np.float32))
    cfg = q.LayerConfig(m=m, base=base, bits_hadamard=9, inner_quant=True, out_type="f32")
    losses = []
    for _ in range(7):
        fwd, sc = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm)
        y = fwd["y"].astype(np.float64)
        losses.append(0.5 * float(((y - y_ref) ** 2).mean()))
        f = lambda name: float(sc[name])
        g = bw.flex_backward((y - y_ref) / y_ref.size, wq.astype(np.float64) * f("s_w"),
                             fwd["X1"].astype(np.float64) * f("s_x1"),
                             fwd["M1"].astype(np.float64) * f("s_m1"),
                             bw.dequantise(fwd["U"], f("s_u")), bw.dequantise(fwd["V"], f("s_v")),
                             fm, xq.shape, m, base)
        for name in ("GP", "BPT", "APT"):
            a, d = getattr(fm, name).astype(np.float64), g["d" + name]
            step = 0.05 * np.abs(a).max() / max(np.abs(d).max(), 1e-30)
            setattr(fm, name, (a - step * d).astype(np.float32))
    assert min(losses[3:]) < 0.6 * losses[0], losses
