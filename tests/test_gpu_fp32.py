"""GPU parity of the fp32 path (bits_in = 32): no casts, float tensors.

Bar: max |y_gpu - y_fp64| <= 1e-4 * max|y_fp64| against the fp64 oracle
(eq. 3 / eq. 4 evaluated in float64 on the same fp32 inputs, and the direct
convolution itself), for every tile size in both bases.  The tensors of the path
are fp32; a Legendre bracket pair (whose factors cancel) is evaluated in double
between its fp32 input and its fp32 result.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import direct, matrices as mx, winograd as wg

pytestmark = pytest.mark.gpu


def run_fp32(x, w, m, base, whole, relu=False):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = x.shape
    K = w.shape[0]
    desc = wn.ConvDesc(N, H, W, C, K, m=m, bits_in=32, relu=int(relu),
                       base=wn.BASE_LEGENDRE if base == "legendre" else wn.BASE_CANONICAL)
    n2, T = desc.n ** 2, desc.tiles
    xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dev)
    wd = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).to(dev)
    y = torch.full((N, H, W, K), 7.0, dtype=torch.float32, device=dev)
    sc = wn.Scales.from_dict({})
    if whole:
        ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        assert ws.numel() >= 4 * n2 * (K * C + T * C + T * K)
        wn.wino_conv2d(desc, xd, wd, y, sc, ws)
    else:
        V = torch.empty((n2, K, C), dtype=torch.float32, device=dev)
        U = torch.empty((n2, T, C), dtype=torch.float32, device=dev)
        M = torch.empty((n2, T, K), dtype=torch.float32, device=dev)
        wn.wino_weight_transform(desc, wd, V, sc)
        wn.wino_input_transform(desc, xd, U, sc)
        wn.wino_contract(desc, U, V, M, sc)
        wn.wino_output_transform(desc, M, y, sc)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("base", ["canonical", "legendre"])
def test_fp32_path_matches_fp64(m, base):
    x, w = si.make_real(3, 9, 7, 48, 80, seed=40 + m)
    mats = mx.Matrices(m, 3)
    ref = (wg.conv_eq4 if base == "legendre" else wg.conv_eq3)(x, w, mats)
    yd = direct.direct_conv(x, w)
    scale = np.abs(yd).max()
    assert np.abs(ref - yd).max() <= 1e-9 * scale
    for whole in (False, True):
        y = run_fp32(x, w, m, base, whole)
        err = np.abs(y - ref).max() / scale
        print("fp32 path F(%d,3) %s whole=%s: rel err %.3g" % (m, base, whole, err))
        assert err <= 1e-4
        assert np.abs(y - yd).max() <= 1e-4 * scale


def test_fp32_path_cfg1_and_relu():
    wl = si.WORKLOADS["cfg1_f2_legendre"]
    x, w = si.make_real(wl.N, wl.H, wl.W, wl.C, wl.K, wl.seed)
    yd = direct.direct_conv(x, w)
    y = run_fp32(x, w, 2, "legendre", True, relu=True)
    assert np.abs(y - np.maximum(yd, 0)).max() <= 1e-4 * np.abs(yd).max()
    assert (y == 0).any() and (y > 0).any()
