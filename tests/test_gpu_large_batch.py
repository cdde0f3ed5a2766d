"""GPU check of the index arithmetic at large tile counts (65536 tiles: the 64x batch that the
benchmark also times).  A batch made of 64 copies of a small batch must give 64 copies of the
small batch's output, bit for bit, on every kernel path; the small batch itself is checked
against the oracle.  The comparison of the large outputs runs on the device (1 GB of fp32 y)."""
import numpy as np
import pytest

import synth_inputs as si
from helpers import assert_layer_parity, oracle_layer

pytestmark = pytest.mark.gpu


def run(desc, x, second, sc, out_dtype):
    import torch
    import paper_2004_11077_amd as wn
    ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=x.device)
    y = torch.empty((desc.N, desc.H, desc.W, desc.K), dtype=out_dtype, device=x.device)
    wn.wino_conv2d(desc, x, second, y, sc, ws)
    torch.cuda.synchronize()
    return y


@pytest.mark.parametrize("name,reps,modes", [
    ("cfg4a_f4_c256", 64, ("off", "on")),        # one kernel per stage; M kept on chip
    ("cfg2_f4_c64", 8, ("on",)),                 # the single kernel, 65536 tiles
])
def test_repeated_batch(name, reps, modes):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    wl = si.WORKLOADS[name]
    L = si.make_layer(wl)
    kw = dict(m=wl.m, base=wl.base, bits_hadamard=wl.bits_hadamard, out_type="f32")
    ora, scd = oracle_layer(L["xq"], L["wq"], L["s_x"], L["s_w"], **kw)
    sc = wn.Scales.from_dict(scd)
    base = wn.BASE_LEGENDRE if wl.base == "legendre" else wn.BASE_CANONICAL
    x1 = torch.from_numpy(L["xq"]).to(dev)
    w = torch.from_numpy(L["wq"]).to(dev)
    xr = x1.repeat(reps, 1, 1, 1).contiguous()
    for mode in modes:
        fused = wn.FUSED_ON if mode == "on" else wn.FUSED_OFF
        common = dict(m=wl.m, base=base, bits_hadamard=wl.bits_hadamard, out_type=wn.OUT_F32,
                      fused=fused)
        small = run(wn.ConvDesc(wl.N, wl.H, wl.W, wl.C, wl.K, **common), x1, w, sc, torch.float32)
        assert_layer_parity(ora, {"y": small.cpu().numpy()}, "f32")
        big_desc = wn.ConvDesc(wl.N * reps, wl.H, wl.W, wl.C, wl.K, **common)
        assert big_desc.tiles == 65536
        big = run(big_desc, xr, w, sc, torch.float32)
        same = (big.view(reps, *small.shape) == small.unsqueeze(0)).all()
        assert bool(same), (name, mode)
        del big
