"""GPU parity of the device-side calibration (wino_calibrate) against the oracle.

The oracle chooses every scale stage after stage as float32(max|real| / qmax)
on the codes the previous stages produced; the library does the same on the
device (exact integer maxima per matrix position, final arithmetic in double on
the host).  Every scale must be the same float32, bit for bit -- then all
downstream codes are identical too, which the test also checks on y.
"""
import numpy as np
import pytest

import synth_inputs as si
from helpers import oracle_layer, small_layer

pytestmark = pytest.mark.gpu


def calibrate_gpu(xq, wq, s_x, s_w, m, base, bits_hadamard, out_type, relu, inner_quant=True):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = xq.shape
    K = wq.shape[0]
    out_id = {"f32": wn.OUT_F32, "i8": wn.OUT_I8}[out_type]
    desc = wn.ConvDesc(N, H, W, C, K, m=m, bits_hadamard=bits_hadamard, out_type=out_id,
                       relu=int(relu), inner_quant=int(inner_quant),
                       base=wn.BASE_LEGENDRE if base == "legendre" else wn.BASE_CANONICAL)
    x = torch.from_numpy(np.ascontiguousarray(xq)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq)).to(dev)
    y = torch.empty((N, H, W, K), dtype=torch.int8 if out_type == "i8" else torch.float32,
                    device=dev)
    ws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    sc = wn.wino_calibrate(desc, x, w, y, float(s_x), float(s_w), ws)
    torch.cuda.synchronize()
    return {name: np.float32(getattr(sc, name)) for name, _ in sc._fields_}, y.cpu().numpy()


def check(xq, wq, s_x, s_w, **kw):
    ora, osc = oracle_layer(xq, wq, s_x, s_w, **kw)
    gsc, y = calibrate_gpu(xq, wq, s_x, s_w, kw["m"], kw["base"], kw.get("bits_hadamard", 8),
                           kw.get("out_type", "f32"), kw.get("relu", False),
                           kw.get("inner_quant", True))
    for name, val in osc.items():
        assert gsc[name] == np.float32(val), (name, gsc[name], val)
    if kw.get("out_type") == "i8":
        assert np.array_equal(y.astype(np.int64), ora["y"])
    else:
        assert np.abs(y - ora["y"]).max() <= 1e-5 * np.abs(ora["y"]).max()


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("base", ["canonical", "legendre"])
def test_calibration_small(m, base):
    xq, wq, s_x, s_w = small_layer(3, 9, 7, 48, 80, seed=80 + m)
    check(xq, wq, s_x, s_w, m=m, base=base, out_type="i8", relu=True)
    check(xq, wq, s_x, s_w, m=m, base=base, bits_hadamard=9, out_type="i8")
    check(xq, wq, s_x, s_w, m=m, base=base, bits_hadamard=32, out_type="f32")


def test_calibration_without_inner_casts_and_all_zero_input():
    xq, wq, s_x, s_w = small_layer(2, 8, 8, 16, 16, seed=90)
    check(xq, wq, s_x, s_w, m=4, base="legendre", inner_quant=False, out_type="i8")
    check(np.zeros_like(xq), wq, np.float32(1.0), s_w, m=4, base="legendre", out_type="i8")


@pytest.mark.parametrize("name", ["cfg1_f2_legendre", "cfg3_f4_c128_h9", "cfg4a_f4_c256"])
def test_calibration_reproduces_the_stored_workload_scales(name):
    wl = si.WORKLOADS[name]
    L = si.make_layer(wl)
    gsc, _ = calibrate_gpu(L["xq"], L["wq"], L["s_x"], L["s_w"], wl.m, wl.base, wl.bits_hadamard,
                           "i8", False)
    stored = si.workload_scales(name)
    for key, val in stored.items():
        assert gsc[key] == np.float32(val), (key, gsc[key], val)
