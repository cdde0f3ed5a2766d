"""Backward pass of the flex layer: library (fp32, through the C ABI) against the fp64 oracle.

The forward tensors handed to the library (U, V, M codes and all scales) are the
ORACLE's forward pass of the same layer (oracle/flex.py, which the forward parity
tests show to be bit-identical to the library's); the library recomputes X1 and M1
from x and M with its exact integer arithmetic.

Tolerance: as for the static backward pass (test_gpu_backward.py) for dM, dU, dV,
dx, dw.  A matrix gradient is a sum over T*C (or T*K, K*C) items of products of
three fp32 factors, accumulated as a fixed tree (lanes, waves, work groups); its
rounding error grows like log2(items) * 2^-24 times the sum of the magnitudes of
the terms, which for these zero-mean terms is about sqrt(items) times the result:
the tests allow 2e-5 of the largest entry of each matrix gradient at up to 10^5
items.
"""
import numpy as np
import pytest

from helpers import small_layer
from oracle import backward as bw
from oracle import flex, quantised as q
from oracle.winograd import extract_tiles
from test_gpu_flex import noisy_matrices

pytestmark = pytest.mark.gpu


def oracle_forward(xq, wq, s_x, s_w, fm, m, base, bits_hadamard):
    cfg = q.LayerConfig(m=m, base=base, bits_hadamard=bits_hadamard, inner_quant=True, out_type="f32")
    return flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm)


def reference(dy, xq, wq, fwd, sc, fm, m, base):
    n = m + 2
    f = lambda name: float(sc[name])
    T = fwd["U"].shape[1]
    K, C = wq.shape[0], wq.shape[1]
    U = bw.dequantise(fwd["U"], f("s_u"))
    V = bw.dequantise(fwd["V"], f("s_v"))
    if base == "legendre":
        X1 = fwd["X1"].astype(np.float64) * f("s_x1")
        M1 = fwd["M1"].astype(np.float64) * f("s_m1")
    else:
        X1 = extract_tiles(xq.astype(np.float64), m, 3) * f("s_x")
        s_m = f("s_m") if "s_m" in sc else f("s_u") * f("s_v")
        M1 = fwd["M"].reshape(n, n, T, K).transpose(2, 0, 1, 3).astype(np.float64) * s_m
    return bw.flex_backward(dy.astype(np.float64), wq.astype(np.float64) * f("s_w"), X1, M1, U, V,
                            fm, xq.shape, m, base)


def run_gpu(dy, xq, wq, fwd, sc, fm, m, base, bits_hadamard):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = xq.shape
    K = wq.shape[0]
    n = m + 2
    desc = wn.ConvDesc(N, H, W, C, K, m=m,
                       base=wn.BASE_LEGENDRE if base == "legendre" else wn.BASE_CANONICAL,
                       bits_hadamard=bits_hadamard)
    n2, T = desc.n ** 2, desc.tiles
    gfm = wn.FlexMatrices(fm.GP, fm.BPT, fm.APT)
    mdt = {8: np.int8, 9: np.int16, 32: np.int32}[bits_hadamard]
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(dev)
    nan = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device=dev)
    dx, dw = nan(N, H, W, C), nan(K, C, 3, 3)
    dGP, dBPT, dAPT = nan(n, 3), nan(n, n), nan(m, n)
    ws = nan(wn.wino_flex_backward_workspace_bytes(desc) // 4)
    scales = {k: float(v) for k, v in sc.items() if k.startswith("s_")}
    wn.wino_flex_backward(desc, gfm, t(dy, np.float32), t(xq, np.int8), t(wq, np.int8),
                          t(fwd["U"], np.int8), t(fwd["V"], np.int8), t(fwd["M"], mdt),
                          wn.Scales.from_dict(scales), dx, dw, dGP, dBPT, dAPT, ws)
    torch.cuda.synchronize()
    r64 = lambda v: (v + 63) // 64 * 64
    out, o = {}, 0
    for name, shp in (("dM", (n2, T, K)), ("dU", (n2, T, C)), ("dV", (n2, K, C))):
        cnt = int(np.prod(shp))
        out[name] = ws[o:o + cnt].reshape(shp).cpu().numpy()
        o += r64(cnt)
    for name, ten in (("dx", dx), ("dw", dw), ("dGP", dGP), ("dBPT", dBPT), ("dAPT", dAPT)):
        out[name] = ten.cpu().numpy()
    return out


def check(ref, got, long_sums=1.0):
    """long_sums: factor on the tolerance of the results summed over all tiles (dV, dw), for
    reductions much longer than the 1024 tiles the plain tolerance was set for."""
    for key, tol in (("dM", 1e-5), ("dU", 1e-5), ("dV", 1e-5 * long_sums), ("dx", 1e-5),
                     ("dw", 1e-5 * long_sums), ("dGP", 2e-5), ("dBPT", 2e-5), ("dAPT", 2e-5)):
        assert got[key].shape == ref[key].shape, key
        assert np.isfinite(got[key]).all(), key + " holds values the kernels did not write"
        bound = tol * max(float(np.abs(ref[key]).max()), 1e-30)
        err = float(np.abs(got[key].astype(np.float64) - ref[key]).max())
        assert err <= bound, "%s: max abs err %g > %g" % (key, err, bound)


CASES = [
    # m, base, (N, H, W, C, K), bits_hadamard
    (4, "legendre", (2, 8, 8, 16, 16), 8),
    (4, "legendre", (3, 11, 6, 48, 80), 9),
    (4, "canonical", (2, 9, 7, 32, 48), 8),
    (4, "canonical", (1, 8, 8, 16, 32), 32),
    (2, "legendre", (2, 7, 9, 32, 16), 8),
    (2, "canonical", (4, 6, 6, 64, 32), 9),
    (6, "legendre", (1, 12, 12, 16, 32), 8),
    (6, "canonical", (2, 7, 8, 32, 16), 8),
    (4, "legendre", (8, 16, 16, 64, 64), 8),      # 128 tiles: several work groups per partial-sum array
    (4, "legendre", (40, 12, 12, 16, 16), 8),     # 360 tiles, few outputs: dV summed from 2 ranges of tiles
    (4, "canonical", (64, 16, 16, 16, 16), 9),    # 1024 tiles: 8 ranges
    (2, "legendre", (64, 16, 16, 16, 16), 8),     # 4096 tiles: 16 ranges, added by a kernel of their own
]


@pytest.mark.parametrize("m,base,shape,bits_hadamard", CASES)
def test_flex_backward_matches_oracle(m, base, shape, bits_hadamard):
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=1300 + m + C)
    fm = noisy_matrices(m, base, seed=17 + m)
    fwd, sc = oracle_forward(xq, wq, s_x, s_w, fm, m, base, bits_hadamard)
    dy = np.random.default_rng(5 + K).standard_normal((N, H, W, K)).astype(np.float32)
    got = run_gpu(dy, xq, wq, fwd, sc, fm, m, base, bits_hadamard)
    T = N * (-(-H // m)) * (-(-W // m))
    check(reference(dy, xq, wq, fwd, sc, fm, m, base), got, long_sums=max(1.0, (T / 1024.0) ** 0.5))


def test_flex_backward_with_static_matrices_matches_static_backward():
    """With the untrained (static) matrices the two backward entry points must agree on dx, dw,
    up to the fp32 rounding of G_P, B_P, A_P themselves (2^-24 relative, amplified by the
    cancellation in the Legendre brackets: a few 1e-5 of the largest gradient)."""
    import torch
    import paper_2004_11077_amd as wn
    m, base, shape = 4, "legendre", (2, 8, 8, 32, 32)
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=77)
    fm = flex.FlexMatrices.from_exact(m, base=base)
    fwd, sc = oracle_forward(xq, wq, s_x, s_w, fm, m, base, 8)
    dy = np.random.default_rng(3).standard_normal((N, H, W, K)).astype(np.float32)
    got = run_gpu(dy, xq, wq, fwd, sc, fm, m, base, 8)
    dev = torch.device("cuda:0")
    desc = wn.ConvDesc(N, H, W, C, K, m=m)
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(dev)
    dx = torch.empty((N, H, W, C), dtype=torch.float32, device=dev)
    dw = torch.empty((K, C, 3, 3), dtype=torch.float32, device=dev)
    ws = torch.empty(wn.wino_backward_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    wn.wino_backward(desc, t(dy, np.float32), t(fwd["U"], np.int8), t(fwd["V"], np.int8),
                     wn.Scales.from_dict({"s_u": float(sc["s_u"]), "s_v": float(sc["s_v"])}), dx, dw, ws)
    torch.cuda.synchronize()
    for name, a, b in (("dx", got["dx"], dx.cpu().numpy()), ("dw", got["dw"], dw.cpu().numpy())):
        err, top = float(np.abs(a - b).max()), float(np.abs(b).max())
        assert err <= 2e-4 * top, "%s: %g vs %g" % (name, err, 2e-4 * top)


def random_cases():
    rng = np.random.default_rng(777)
    out = []
    for i in range(10):
        m = int(rng.choice([2, 4, 6]))
        out.append((m, str(rng.choice(["canonical", "legendre"])),
                    (int(rng.integers(1, 4)), int(rng.integers(1, 13)), int(rng.integers(1, 13)),
                     int(rng.choice([16, 32, 48, 80])), int(rng.choice([16, 32, 48, 80]))),
                    int(rng.choice([8, 9, 32]))))
    return out


@pytest.mark.parametrize("m,base,shape,bits_hadamard", random_cases())
def test_flex_backward_random_shapes(m, base, shape, bits_hadamard):
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=2100 + m + C + H)
    fm = noisy_matrices(m, base, seed=29 + m)
    fwd, sc = oracle_forward(xq, wq, s_x, s_w, fm, m, base, bits_hadamard)
    dy = np.random.default_rng(11 + K + W).standard_normal((N, H, W, K)).astype(np.float32)
    got = run_gpu(dy, xq, wq, fwd, sc, fm, m, base, bits_hadamard)
    check(reference(dy, xq, wq, fwd, sc, fm, m, base), got)
