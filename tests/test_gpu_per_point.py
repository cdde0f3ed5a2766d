"""Per-Winograd-point scales (U and V: one scale per point; M: power-of-two refinements of
s_m) on the GPU against the oracle: every integer tensor bit-exact, fp32 output within 1e-5
of the output range, device-side calibration identical to the oracle's."""
import numpy as np
import pytest

import synth_inputs as si
from helpers import assert_layer_parity, gpu_layer, oracle_layer, small_layer

pytestmark = pytest.mark.gpu

CASES = [
    # m, base, (N, H, W, C, K), bits_hadamard, out_type, relu, whole
    (2, "canonical", (2, 8, 8, 16, 16), 8, "f32", False, False),
    (2, "legendre", (1, 7, 9, 32, 48), 9, "i8", True, True),
    (4, "canonical", (2, 8, 8, 64, 32), 8, "f32", True, True),
    (4, "canonical", (3, 10, 6, 48, 80), 9, "i8", False, False),
    (4, "legendre", (2, 8, 8, 32, 64), 8, "f32", False, False),
    (4, "legendre", (1, 13, 5, 256, 256), 8, "i8", True, True),
    (6, "canonical", (1, 12, 12, 16, 32), 8, "f32", False, True),
    (6, "legendre", (2, 7, 8, 32, 16), 9, "i8", True, False),
]


@pytest.mark.parametrize("m,base,shape,bh,out_type,relu,whole", CASES)
def test_per_point_layer_matches_the_oracle(m, base, shape, bh, out_type, relu, whole):
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=400 + m + C, outliers=0.01)
    kw = dict(m=m, base=base, bits_hadamard=bh, out_type=out_type, relu=relu, per_point=True)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    assert np.shape(sc["s_u"]) == (m + 2, m + 2)
    assert m == 2 or max(sc["m_shift"]) > 0          # F(2,3) points have similar ranges
    got = gpu_layer(xq, wq, sc, whole=whole, **kw)
    assert_layer_parity(ora, got, out_type)


@pytest.mark.parametrize("m,base,shape,bh,out_type,relu", [
    (4, "canonical", (2, 8, 8, 64, 64), 8, "f32", False),      # one channel chunk
    (4, "legendre", (3, 9, 7, 48, 80), 9, "i8", True),
    (4, "canonical", (1, 8, 8, 144, 32), 8, "i8", True),        # several channel chunks
    (2, "legendre", (2, 6, 6, 32, 16), 8, "f32", False),
])
def test_fused_variant_with_per_point_scales(m, base, shape, bh, out_type, relu):
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=600 + m + C, outliers=0.01)
    kw = dict(m=m, base=base, bits_hadamard=bh, out_type=out_type, relu=relu, per_point=True)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got = gpu_layer(xq, wq, sc, fused=True, **kw)
    assert_layer_parity(ora, got, out_type)


def test_per_point_on_the_benchmark_layer_is_far_more_accurate():
    """cfg4a shape with a smaller batch, canonical base: the reason the option exists."""
    from oracle import direct
    wl = si.WORKLOADS["cfg4a_f4_c256"]
    x, w = si.make_real(16, wl.H, wl.W, wl.C, wl.K, wl.seed, wl.outliers)
    xq, s_x = si.cast_int8(x)
    wq, s_w = si.cast_int8(w)
    yd = direct.direct_conv(xq * float(s_x), wq * float(s_w))
    err = {}
    for pp in (False, True):
        kw = dict(m=4, base="canonical", per_point=pp)
        ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
        got = gpu_layer(xq, wq, sc, whole=True, **kw)
        assert_layer_parity(ora, got)
        err[pp] = float(np.sqrt(np.mean((got["y"] - yd) ** 2)) / np.sqrt(np.mean(yd ** 2)))
    assert err[True] < err[False] / 8, err


@pytest.mark.parametrize("m,base,bh,out_type,relu", [(4, "canonical", 8, "i8", True),
                                                     (4, "legendre", 9, "f32", False),
                                                     (2, "legendre", 8, "i8", False),
                                                     (6, "canonical", 8, "f32", True)])
def test_per_point_calibration_equals_the_oracles(m, base, bh, out_type, relu):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K = 2, 9, 8, 32, 48
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=500 + m)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, m=m, base=base, bits_hadamard=bh, out_type=out_type,
                           relu=relu, per_point=True)
    desc = wn.ConvDesc(N, H, W, C, K, m=m,
                       base=wn.BASE_LEGENDRE if base == "legendre" else wn.BASE_CANONICAL,
                       bits_hadamard=bh, out_type=wn.OUT_I8 if out_type == "i8" else wn.OUT_F32,
                       relu=int(relu))
    x = torch.from_numpy(np.ascontiguousarray(xq, dtype=np.int8)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq, dtype=np.int8)).to(dev)
    y = torch.zeros((N, H, W, K), dtype=torch.int8 if out_type == "i8" else torch.float32,
                    device=dev)
    cws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    got = wn.wino_calibrate(desc, x, w, y, float(s_x), float(s_w), cws, per_point=True)
    torch.cuda.synchronize()
    gd = got.to_dict(m + 2)
    for name, val in sc.items():
        if name in ("s_u", "s_v"):
            assert np.array_equal(np.asarray(gd[name], dtype=np.float32),
                                  np.asarray(val, dtype=np.float32)), name
        elif name == "m_shift":
            assert list(gd[name]) == [int(v) for v in val]
        else:
            assert np.float32(gd[name]) == np.float32(val), name
    if out_type == "i8":
        assert np.array_equal(y.cpu().numpy().astype(np.int64), ora["y"])
    else:
        ref = ora["y"]
        assert float(np.abs(y.cpu().numpy() - ref).max()) <= 1e-5 * float(np.abs(ref).max())
