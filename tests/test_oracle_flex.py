"""Pins for oracle/flex.py (the layer with run-time fp32 matrices, Section 4.2 "flex").

Independent of the module's own formulas:

* the fp32 bracket against explicit scalar loops on one tile and against a float64
  ``T @ X @ T.T`` with a non-symmetric random matrix (orientation, index order);
* matrices whose fp32 arithmetic is exact (integers and dyadic fractions: the
  canonical F(2,3) set, and B^T / A^T of canonical F(4,3)) must reproduce the static
  quantised layer bit for bit;
* the static rational matrices rounded to fp32 must give codes that differ from the
  static layer's by at most one step, and rarely (near-ties only);
* with arbitrary perturbed matrices the layer must converge, as the bit width grows, to
  a float64 evaluation of the formula of eq. 3 / eq. 4 with those same matrices.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import flex, matrices as mx, quantised as q
from oracle.winograd import extract_tiles, scatter_tiles


def tiny(N=1, H=8, W=8, C=16, K=16, seed=0, bits=8):
    x, w = si.make_real(N, H, W, C, K, seed)
    xq, s_x = q.quantise_real(x, bits)
    wq, s_w = q.quantise_real(w, bits)
    return xq, wq, s_x, s_w


def test_fsandwich_against_scalar_loops_and_float64():
    rng = np.random.default_rng(0)
    Tm = rng.standard_normal((6, 4)).astype(np.float32)          # non-square, non-symmetric
    X = rng.integers(-127, 128, size=(3, 4, 4, 2))
    got = flex.fsandwich(Tm, X)
    assert got.shape == (3, 6, 6, 2) and got.dtype == np.float32
    for t in range(3):
        for c in range(2):
            ref64 = Tm.astype(np.float64) @ X[t, :, :, c].astype(np.float64) @ Tm.astype(np.float64).T
            assert np.allclose(got[t, :, :, c], ref64, rtol=1e-5, atol=1e-3)
            for i in range(6):
                left = []
                for b in range(4):
                    acc = np.float32(Tm[i, 0] * np.float32(X[t, 0, b, c]))
                    for a in range(1, 4):
                        acc = np.float32(acc + np.float32(Tm[i, a] * np.float32(X[t, a, b, c])))
                    left.append(acc)
                for j in range(6):
                    acc = np.float32(left[0] * Tm[j, 0])
                    for b in range(1, 4):
                        acc = np.float32(acc + np.float32(left[b] * Tm[j, b]))
                    assert acc == got[t, i, j, c]


def test_fcast_is_the_single_rounding_cast():
    val = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 1e9, -1e9, 126.5, 127.49], dtype=np.float32)
    got = flex.fcast(val, 1.0, 1.0, 127)
    assert got.tolist() == [0, 2, 2, 0, -2, 127, -127, 126, 127]


@pytest.mark.parametrize("out_type", ["f32", "i8"])
def test_exact_fp32_matrices_reproduce_the_static_layer_F2(out_type):
    """Canonical F(2,3): G has only 1 and +-1/2, B^T and A^T are integer, so every fp32
    bracket is exact and the flex layer must equal the static one bit for bit."""
    xq, wq, s_x, s_w = tiny(N=2, H=6, W=6, seed=3)
    cfg = q.LayerConfig(m=2, base="canonical", out_type=out_type, relu=True)
    ref, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    fm = flex.FlexMatrices.from_exact(2, base="canonical")
    got, _ = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm, scales=sc)
    for key in ("V", "U", "M"):
        assert np.array_equal(got[key], ref[key]), key
    if out_type == "i8":
        assert np.array_equal(got["y"], ref["y"])
    else:
        assert np.allclose(got["y"], ref["y"], rtol=1e-6, atol=0)
    # and its own calibration lands on the same scales
    _, sc2 = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm)
    for name in ("s_u", "s_v", "s_m") + (("s_y",) if out_type == "i8" else ()):
        assert np.isclose(float(sc2[name]), float(sc[name]), rtol=1e-6), name


def test_integer_brackets_of_canonical_F4_are_exact_and_G_is_near():
    xq, wq, s_x, s_w = tiny(seed=4)
    cfg = q.LayerConfig(m=4, base="canonical", out_type="i8")
    ref, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    fm = flex.FlexMatrices.from_exact(4, base="canonical")
    got, _ = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm, scales=sc)
    assert np.array_equal(got["U"], ref["U"])                     # B^T is an integer matrix
    dv = np.abs(got["V"] - ref["V"])
    assert dv.max() <= 1 and np.mean(dv != 0) < 0.01              # G has thirds: near-ties only
    # output bracket alone, fed with the static layer's M: A^T is an integer matrix
    n, m = 6, 4
    T, K = ref["M"].shape[1:]
    cur = ref["M"].reshape(n, n, T, K).transpose(2, 0, 1, 3)
    val = flex.fsandwich(fm.APT, cur)
    assert np.array_equal(val.astype(np.int64), ref["Y_num"])


def test_rounded_static_legendre_matrices_stay_within_one_step():
    xq, wq, s_x, s_w = tiny(seed=5)
    cfg = q.LayerConfig(m=4, base="legendre", out_type="i8")
    ref, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    fm = flex.FlexMatrices.from_exact(4, base="legendre")
    got, _ = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm, scales=sc)
    assert np.array_equal(got["X1"], ref["X1"])                   # integer bracket, same code path
    for key in ("W1", "U"):
        d = np.abs(got[key] - ref[key])
        assert d.max() <= 1 and np.mean(d != 0) < 0.02, key


def formula_fp64(xq, wq, s_x, s_w, m, base, fm):
    """eq. 3 / eq. 4 with the given real matrices, no cast anywhere, float64."""
    mats = mx.Matrices(m, 3)
    f64 = lambda Tm: np.array([[float(v) for v in row] for row in Tm])
    G, BT, AT = (np.asarray(a, dtype=np.float64) for a in (fm.GP, fm.BPT, fm.APT))
    x = xq.astype(np.float64) * float(s_x)
    w = wq.astype(np.float64) * float(s_w)
    N, H, W, C = x.shape
    d = extract_tiles(x, m, 3)
    Wt = np.einsum("ia,kcab,jb->kcij", G, w, G)
    if base == "legendre":
        PinvT, Pinv = f64(mats.PinvT), f64(mats.Pinv)
        Wt = np.einsum("ia,kcab,bj->kcij", Pinv, Wt, PinvT)
        d = np.einsum("ia,tabc,bj->tijc", PinvT, d, Pinv)
    U = np.einsum("ia,tabc,jb->tijc", BT, d, BT)
    M = np.einsum("tijc,kcij->tijk", U, Wt)
    if base == "legendre":
        M = np.einsum("ia,tabk,bj->tijk", PinvT, M, Pinv)
    Y = np.einsum("ia,tabk,jb->tijk", AT, M, AT)
    return scatter_tiles(Y, N, H, W, m)


@pytest.mark.parametrize("m,base", [(2, "canonical"), (4, "canonical"), (4, "legendre"),
                                    (6, "legendre")])
def test_converges_to_the_fp64_formula_with_arbitrary_matrices(m, base):
    rng = np.random.default_rng(10 * m)
    fm = flex.FlexMatrices.from_exact(m, base=base)
    for name in ("GP", "BPT", "APT"):
        a = getattr(fm, name)
        noise = (0.05 * rng.standard_normal(a.shape) * np.abs(a).max()).astype(np.float32)
        setattr(fm, name, (a + noise).astype(np.float32))         # dense, non-symmetric
    errs = []
    for bits in (10, 13, 16):
        xq, wq, s_x, s_w = tiny(N=1, H=7, W=9, C=8, K=8, seed=6, bits=bits)
        cfg = q.LayerConfig(m=m, base=base, bits=bits, bits_hadamard=32)
        got, _ = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm)
        ref = formula_fp64(xq, wq, s_x, s_w, m, base, fm)
        errs.append(float(np.abs(got["y"] - ref).max() / np.abs(ref).max()))
    assert errs[2] < errs[1] < errs[0], errs
    assert errs[2] < errs[0] / 16, errs                           # ~ 2^-bits
    assert errs[2] < 2e-2, errs
