"""Pins for oracle/quantised.py.

The paper prints no worked numeric example of the quantised pipeline (its
quantisation figure is missing), so the absolute quantised outputs are
"parity unpinned" by the paper.  What is pinned here, independently of the
oracle's own formulas:

* the integer transform of the canonical input stage, recomputed from
  polynomial coefficients obtained with numpy.poly and rounded in exact
  rational arithmetic;
* the fp32 rounding rule against exact-rational round-half-even (they may
  differ only at near-ties, which are counted);
* convergence of the whole quantised layer to the direct convolution as the
  bit width grows (catches any scale, index, transpose or layout mistake);
* the collapse of eq. 4 to eq. 3 without inner casts;
* an a-priori worst-case error bound, and monotonicity in the Hadamard bits.
"""
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs as si
from oracle import direct, matrices as mx, quantised as q, winograd as wg


def tiny_layer(N=1, H=8, W=8, C=16, K=16, seed=0, bits=8, outliers=0.0):
    x, w = si.make_real(N, H, W, C, K, seed, outliers)
    xq, s_x = q.quantise_real(x, bits)
    wq, s_w = q.quantise_real(w, bits)
    return x, w, xq, wq, s_x, s_w


def exact_round_half_even(v):
    """Round a Fraction to the nearest integer, ties to even."""
    fl = v.numerator // v.denominator
    rem = v - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def test_generator_cast_agrees_with_oracle_cast():
    wl = si.WORKLOADS["cfg1_f2_legendre"]
    L = si.make_layer(wl)
    xq, s_x = q.quantise_real(L["x"], 8)
    wq, s_w = q.quantise_real(L["w"], 8)
    assert np.array_equal(xq, L["xq"]) and s_x == L["s_x"]
    assert np.array_equal(wq, L["wq"]) and s_w == L["s_w"]
    assert L["xq"].min() >= -127 and L["wq"].min() >= -127


@pytest.mark.parametrize("m", [2, 4])
def test_canonical_U_against_numpy_poly_and_exact_rounding(m):
    pts = [float(p) for p in mx.POINTS[m]]
    n = m + 2
    # rows of B^T from a library routine: coefficients of prod_{k != j}(x - p_k)
    BT = np.zeros((n, n), dtype=np.int64)
    for j in range(n - 1):
        coef = np.poly([p for k, p in enumerate(pts) if k != j])[::-1]     # ascending
        BT[j, :len(coef)] = np.rint(coef).astype(np.int64)
    BT[n - 1, :] = np.rint(np.poly(pts)[::-1]).astype(np.int64)

    _, _, xq, wq, s_x, s_w = tiny_layer(1, 8, 8, 4, 4, seed=3)
    cfg = q.LayerConfig(m=m, base="canonical")
    out, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    TH = TW = 8 // m
    ratio = Fraction(float(sc["s_x"])) / Fraction(float(sc["s_u"]))
    near_ties = 0
    for ty in range(TH):
        for tx in range(TW):
            t = ty * TW + tx
            for c in range(4):
                X = np.zeros((n, n), dtype=np.int64)
                for a in range(n):
                    for b in range(n):
                        hh, ww = ty * m - 1 + a, tx * m - 1 + b
                        if 0 <= hh < 8 and 0 <= ww < 8:
                            X[a, b] = xq[0, hh, ww, c]
                num = BT @ X @ BT.T
                for i in range(n):
                    for j in range(n):
                        exact = Fraction(int(num[i, j])) * ratio
                        want = max(-127, min(127, exact_round_half_even(exact)))
                        got = int(out["U"][i * n + j, t, c])
                        if got != want:
                            frac = exact - (exact.numerator // exact.denominator)
                            assert abs(frac - Fraction(1, 2)) < Fraction(1, 1000)
                            assert abs(got - want) == 1
                            near_ties += 1
    assert near_ties <= 2


def test_fp32_rounding_rule_vs_exact_rational_on_legendre_stage():
    _, _, xq, wq, s_x, s_w = tiny_layer(1, 8, 8, 8, 8, seed=4)
    cfg = q.LayerConfig(m=4, base="legendre")
    out, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    sm = q.StageMatrices(cfg)
    Nm, rho = sm.in_outer
    num = q.sandwich_tiles(Nm, out["X1"])                   # [T,6,6,C]
    U = out["U"].reshape(6, 6, num.shape[0], num.shape[3]).transpose(2, 0, 1, 3)
    s_prev, s_next = Fraction(float(sc["s_x1"])), Fraction(float(sc["s_u"]))
    diff = 0
    for idx in np.ndindex(*num.shape):
        i, j = idx[1], idx[2]
        exact = Fraction(int(num[idx])) * s_prev / (rho[i] * rho[j] * s_next)
        want = max(-127, min(127, exact_round_half_even(exact)))
        if want != int(U[idx]):
            frac = exact - (exact.numerator // exact.denominator)
            assert abs(frac - Fraction(1, 2)) < Fraction(1, 1000)
            diff += 1
    assert diff <= num.size // 1000 + 1


def test_requant_ties_to_even_and_clamp():
    num = np.array([[[[1], [3]], [[5], [-1]]]], dtype=np.int64)      # [T=1,2,2,C=1]
    mult = np.full((2, 2), 0.5, dtype=np.float32)
    got = q.requant(num, mult, 127, (1, 2)).reshape(-1).tolist()
    assert got == [0, 2, 2, 0]                   # 0.5->0, 1.5->2, 2.5->2, -0.5->-0
    big = np.array([[[[1000], [-1000]], [[254], [-255]]]], dtype=np.int64)
    got = q.requant(big, mult, 127, (1, 2)).reshape(-1).tolist()
    assert got == [127, -127, 127, -127]         # symmetric clamp, never -128


def test_mult_table_formula():
    tab = q.mult_table([3, 5], [3, 5], np.float32(0.1), np.float32(0.7))
    assert tab.dtype == np.float32
    want = np.float32(float(np.float32(0.1)) / (15.0 * float(np.float32(0.7))))
    assert tab[0, 1] == want and tab[1, 0] == want


def test_all_zero_tensor_gives_unit_scales_and_zero_output():
    xq = np.zeros((1, 4, 4, 2), dtype=np.int64)
    wq = np.ones((2, 2, 3, 3), dtype=np.int64)
    out, sc = q.run_layer(xq, wq, np.float32(1.0), np.float32(0.5), q.LayerConfig(m=4))
    assert sc["s_u"] == 1.0 and sc["s_m"] == 1.0 and sc["s_x1"] == 1.0
    assert np.all(out["y"] == 0)


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("base", ["canonical", "legendre"])
def test_converges_to_direct_convolution_with_bit_width(m, base):
    x, w = si.make_real(1, 8, 8, 8, 8, seed=1)
    yd = direct.direct_conv(x, w)
    rms = np.sqrt(np.mean(yd ** 2))
    errs = []
    for bits in (10, 14, 18, 22):
        xq, s_x = q.quantise_real(x, bits)
        wq, s_w = q.quantise_real(w, bits)
        cfg = q.LayerConfig(m=m, base=base, bits=bits, bits_hadamard=bits)
        out, _ = q.run_layer(xq, wq, s_x, s_w, cfg)
        errs.append(np.sqrt(np.mean((out["y"] - yd) ** 2)) / rms)
    # each 4 extra bits must buy about 16x; the fp32 multiplier (2^-24) is the floor
    assert errs[1] < errs[0] / 8 and errs[2] < errs[1] / 8 and errs[3] < errs[2] / 4
    assert errs[3] < 2e-3 if m < 6 else errs[3] < 5e-2


@pytest.mark.parametrize("base", ["chebyshev", "hermite"])
def test_other_bases_converge_and_collapse_without_inner_casts(base):
    """The alternatives Section 4.1 names run through the same two-bracket pipeline."""
    x, w = si.make_real(1, 8, 8, 8, 8, seed=1)
    yd = direct.direct_conv(x, w)
    rms = np.sqrt(np.mean(yd ** 2))
    errs = []
    for bits in (14, 18, 22):
        xq, s_x = q.quantise_real(x, bits)
        wq, s_w = q.quantise_real(w, bits)
        out, _ = q.run_layer(xq, wq, s_x, s_w,
                             q.LayerConfig(m=4, base=base, bits=bits, bits_hadamard=bits))
        errs.append(np.sqrt(np.mean((out["y"] - yd) ** 2)) / rms)
    assert errs[1] < errs[0] / 8 and errs[2] < errs[1] / 4, errs
    _, _, xq, wq, s_x, s_w = tiny_layer(1, 8, 8, 4, 4, seed=2)
    can, _ = q.run_layer(xq, wq, s_x, s_w, q.LayerConfig(m=4, base="canonical"))
    col, _ = q.run_layer(xq, wq, s_x, s_w, q.LayerConfig(m=4, base=base, inner_quant=False))
    for key in ("U", "V", "M", "y"):
        assert np.array_equal(can[key], col[key])


@pytest.mark.parametrize("m", [2, 4, 6])
def test_no_inner_casts_collapses_legendre_to_canonical(m):
    _, _, xq, wq, s_x, s_w = tiny_layer(1, 8, 8, 4, 4, seed=2)
    can, sc_c = q.run_layer(xq, wq, s_x, s_w, q.LayerConfig(m=m, base="canonical"))
    leg, sc_l = q.run_layer(xq, wq, s_x, s_w,
                            q.LayerConfig(m=m, base="legendre", inner_quant=False))
    for key in ("U", "V", "M", "Y_num"):
        assert np.array_equal(can[key], leg[key])
    assert np.array_equal(can["y"], leg["y"])
    assert sc_c == sc_l
    # with inner casts the codes do differ (the base change is not a no-op)
    leg2, _ = q.run_layer(xq, wq, s_x, s_w, q.LayerConfig(m=m, base="legendre"))
    assert not np.array_equal(can["U"], leg2["U"])


def test_contraction_against_explicit_loops():
    rng = np.random.default_rng(8)
    U = rng.integers(-127, 128, size=(4, 3, 5))
    V = rng.integers(-127, 128, size=(4, 2, 5))
    sc = {"s_u": np.float32(0.01), "s_v": np.float32(0.02)}
    out = {}
    M, _ = q.contraction(U, V, q.LayerConfig(bits_hadamard=32), sc, out)
    for p in range(4):
        for t in range(3):
            for k in range(2):
                assert M[p, t, k] == sum(int(U[p, t, c]) * int(V[p, k, c]) for c in range(5))
    Mq, s_m = q.contraction(U, V, q.LayerConfig(bits_hadamard=9), sc, out)
    assert np.abs(Mq).max() == 255
    assert s_m == np.float32(np.abs(M).max() * (float(sc["s_u"]) * float(sc["s_v"])) / 255)


def test_given_scales_reproduce_calibrated_run():
    _, _, xq, wq, s_x, s_w = tiny_layer(1, 8, 8, 4, 4, seed=9)
    cfg = q.LayerConfig(m=4, base="legendre", bits_hadamard=9, out_type="i8", relu=True)
    a, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    b, sc2 = q.run_layer(xq, wq, s_x, s_w, cfg, scales=sc)
    assert sc == sc2
    for key in ("X1", "U", "W1", "V", "M", "M1", "y"):
        assert np.array_equal(a[key], b[key])
    assert a["y"].min() >= 0 and a["y"].max() == 127
    assert np.abs(a["y"] * float(sc["s_y"]) - a["y_real"]).max() <= float(sc["s_y"]) * 0.5001


def test_integer_output_canonical():
    _, _, xq, wq, s_x, s_w = tiny_layer(1, 8, 8, 4, 4, seed=9)
    cfg = q.LayerConfig(m=4, base="canonical", out_type="i32")
    a, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    f, _ = q.run_layer(xq, wq, s_x, s_w, q.LayerConfig(m=4, base="canonical"))
    assert np.allclose(a["y"] * float(sc["s_m"]), f["y"], rtol=1e-12)


def _norm(T):
    return max(sum(abs(v) for v in row) for row in T)


def winograd_error_bound(x, w, cfg, sc):
    """Worst-case |y_q - y_exact|: every cast adds at most half a step, pushed
    through the max-abs-row-sum norms of the remaining linear maps and through
    the channel sum of the element-wise products."""
    M = mx.Matrices(cfg.m, cfg.r)
    C = x.shape[-1]
    f = lambda T: float(_norm(T)) ** 2
    e_x, e_w = float(sc["s_x"]) / 2, float(sc["s_w"]) / 2
    if cfg.base == "legendre":
        e_x1 = f(M.PinvT) * e_x + float(sc["s_x1"]) / 2
        e_u = f(M.BPT) * e_x1 + float(sc["s_u"]) / 2
        e_w1 = f(M.GP) * e_w + float(sc["s_w1"]) / 2
        e_v = f(M.Pinv) * e_w1 + float(sc["s_v"]) / 2
    else:
        e_u = f(M.BT) * e_x + float(sc["s_u"]) / 2
        e_v = f(M.G) * e_w + float(sc["s_v"]) / 2
    BT = np.array([[float(v) for v in r] for r in M.BT])
    G = np.array([[float(v) for v in r] for r in M.G])
    u_max = np.abs(np.einsum("ia,tabc,jb->tijc", BT, wg.extract_tiles(x, cfg.m, cfg.r), BT)).max()
    v_max = np.abs(np.einsum("ia,kcab,jb->kcij", G, w, G)).max()
    e_m = C * (u_max * e_v + (v_max + e_v) * e_u)
    if cfg.bits_hadamard != 32:
        e_m += float(sc["s_m"]) / 2
    if cfg.base == "legendre":
        e_m1 = f(M.PinvT) * e_m + float(sc["s_m1"]) / 2
        return f(M.APT) * e_m1
    return f(M.AT) * e_m


@pytest.mark.parametrize("base", ["canonical", "legendre"])
def test_error_bounds_and_hadamard_bit_monotonicity(base):
    x, w, xq, wq, s_x, s_w = tiny_layer(2, 8, 8, 16, 16, seed=0)
    x, w = x.astype(np.float64), w.astype(np.float64)
    yd = direct.direct_conv(x, w)
    # quantised direct convolution and its own worst-case bound
    yq = direct.direct_conv(xq, wq, dtype=np.int64) * (float(s_x) * float(s_w))
    C = x.shape[-1]
    bound_d = 9 * C * (np.abs(x).max() * float(s_w) / 2 + np.abs(w).max() * float(s_x) / 2
                       + float(s_x) * float(s_w) / 4)
    assert np.abs(yq - yd).max() <= bound_d
    rms = {}
    for bh in (8, 9, 32):
        cfg = q.LayerConfig(m=4, base=base, bits_hadamard=bh)
        out, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
        err = np.abs(out["y"] - yd)
        assert err.max() <= winograd_error_bound(x, w, cfg, sc)
        rms[bh] = np.sqrt(np.mean(err ** 2))
    assert rms[32] <= rms[9] <= rms[8]
    assert np.sqrt(np.mean((yq - yd) ** 2)) < rms[32]       # direct int8 is the more accurate one


# ---- per-point operand scales (an option of dynamic quantisation, not in the paper) ------

def test_per_point_scales_all_equal_reproduce_the_per_tensor_layer():
    _, _, xq, wq, s_x, s_w = tiny_layer(2, 7, 6, 8, 8, seed=8)
    for base in ("canonical", "legendre"):
        ref, sc = q.run_layer(xq, wq, s_x, s_w, q.LayerConfig(m=4, base=base, out_type="i8"))
        flat = dict(sc)
        flat["s_u"] = np.full((6, 6), sc["s_u"], dtype=np.float32)
        flat["s_v"] = np.full((6, 6), sc["s_v"], dtype=np.float32)
        flat["m_shift"] = np.zeros(36, dtype=np.int64)
        got, _ = q.run_layer(xq, wq, s_x, s_w,
                             q.LayerConfig(m=4, base=base, out_type="i8", per_point=True), scales=flat)
        for key in ("U", "V", "M", "y"):
            assert np.array_equal(got[key], ref[key]), (base, key)


def test_per_point_U_against_exact_rational_rounding():
    """Each point's codes are the exactly rounded real values over that point's own scale."""
    _, _, xq, wq, s_x, s_w = tiny_layer(1, 8, 8, 8, 8, seed=9)
    cfg = q.LayerConfig(m=4, base="canonical", per_point=True)
    out, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    assert np.shape(sc["s_u"]) == (6, 6) and np.shape(sc["s_v"]) == (6, 6)
    assert len(set(np.asarray(sc["s_u"]).ravel().tolist())) > 10      # really per point
    BT = mx.Matrices(4, 3).BT
    d = wg.extract_tiles(xq.astype(np.int64), 4, 3)                   # [T,6,6,C]
    T, C = d.shape[0], d.shape[3]
    U = out["U"].reshape(6, 6, T, C)
    near = 0
    for t in range(0, T, 2):
        for c in range(0, C, 3):
            X = [[Fraction(int(d[t, a, b, c])) for b in range(6)] for a in range(6)]
            R = mx.matmul(mx.matmul(BT, X), mx.transpose(BT))
            for i in range(6):
                for j in range(6):
                    exact = R[i][j] * Fraction(float(s_x)) / Fraction(float(sc["s_u"][i][j]))
                    want = max(-127, min(127, exact_round_half_even(exact)))
                    if want != int(U[i, j, t, c]):
                        frac = exact - (exact.numerator // exact.denominator)
                        assert abs(frac - Fraction(1, 2)) < Fraction(1, 1000)
                        near += 1
    assert near <= 3
    # every point uses its full range
    assert np.all(np.abs(out["U"]).reshape(36, -1).max(axis=1) == 127)


@pytest.mark.parametrize("base", ["canonical", "legendre"])
def test_per_point_layer_converges_and_is_at_least_as_accurate(base):
    x, w = si.make_real(1, 8, 8, 8, 8, seed=1)
    yd = direct.direct_conv(x, w)
    rms = np.sqrt(np.mean(yd ** 2))
    errs = []
    for bits in (10, 14, 18):
        xq, s_x = q.quantise_real(x, bits)
        wq, s_w = q.quantise_real(w, bits)
        cfg = q.LayerConfig(m=4, base=base, bits=bits, bits_hadamard=bits + 8, per_point=True)
        out, _ = q.run_layer(xq, wq, s_x, s_w, cfg)
        errs.append(float(np.sqrt(np.mean((out["y"] - yd) ** 2)) / rms))
    assert errs[0] > 8 * errs[1] > 64 * errs[2], errs
    # at 8 bits (9-bit Hadamard stage) per-point scales must not lose to per-tensor ones
    xq, s_x = q.quantise_real(x, 8)
    wq, s_w = q.quantise_real(w, 8)
    e = {}
    for pp in (False, True):
        out, _ = q.run_layer(xq, wq, s_x, s_w,
                             q.LayerConfig(m=4, base=base, bits_hadamard=9, per_point=pp))
        e[pp] = float(np.sqrt(np.mean((out["y"] - yd) ** 2)) / rms)
    assert e[True] < e[False], e
    if base == "canonical":
        assert e[True] < e[False] / 8, e          # the point of it: an order of magnitude


def test_per_point_M_shifts_are_the_largest_that_do_not_clip():
    _, _, xq, wq, s_x, s_w = tiny_layer(2, 8, 8, 16, 16, seed=12)
    cfg = q.LayerConfig(m=4, base="canonical", per_point=True)
    out, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    shift = np.asarray(sc["m_shift"])
    assert shift.shape == (36,) and shift.min() == 0 and 0 < shift.max() <= 8
    s_uv = (np.asarray(sc["s_u"], dtype=np.float64) * np.asarray(sc["s_v"], dtype=np.float64)).reshape(36)
    for p in range(36):
        real = np.abs(out["M_acc"][p]).max() * s_uv[p]             # largest real value of point p
        step = float(sc["s_m"]) / 2.0 ** shift[p]
        assert real <= 127 * step * (1 + 1e-6)                      # not clipped
        if shift[p] < 8:
            assert real > 127 * step / 2 * (1 - 1e-6)               # one more bit would clip
        # stored codes are the real values over the point's own step, exactly rounded
        # except at near-ties
        want = np.clip(np.rint(out["M_acc"][p] * s_uv[p] / step), -127, 127)
        d = np.abs(want - out["M"][p])
        assert d.max() <= 1 and np.mean(d != 0) < 0.01
    # reconstruction: what the output bracket receives, times its scale, is M within half a step
    smax = shift.max()
    fed = out["M"] * (2 ** (smax - shift)).reshape(36, 1, 1)
    real_all = out["M_acc"] * s_uv.reshape(36, 1, 1)
    err = np.abs(fed * (float(sc["s_m"]) / 2.0 ** smax) - real_all)
    half = (float(sc["s_m"]) / 2.0 ** shift / 2).reshape(36, 1, 1)
    assert np.all(err <= half * (1 + 1e-5))


def test_per_point_needs_a_cast_of_the_contraction_result():
    _, _, xq, wq, s_x, s_w = tiny_layer(seed=3)
    with pytest.raises(AssertionError):
        q.run_layer(xq, wq, s_x, s_w, q.LayerConfig(m=4, bits_hadamard=32, per_point=True))
