"""GPU parity of the fused variant (one kernel: input transform, contraction,
output transform; U and M never leave the chip) against the CPU oracle.

Only V and y are observable: V and int8 outputs must be bit-exact, fp32 outputs
within 1e-5 * max|y_oracle|.  Because every intermediate code feeds the next
integer stage, an int8 output that matches bit for bit also pins U and M.
"""
import numpy as np
import pytest

import synth_inputs as si
from helpers import assert_layer_parity, gpu_layer, oracle_layer, small_layer

pytestmark = pytest.mark.gpu


def run_fused(xq, wq, s_x, s_w, **kw):
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got = gpu_layer(xq, wq, sc, fused=True, **kw)
    assert_layer_parity(ora, got, kw.get("out_type", "f32"))
    return got, sc


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("base", ["canonical", "legendre"])
@pytest.mark.parametrize("bits_hadamard", [8, 9])
def test_fused_small_ragged(m, base, bits_hadamard):
    # 3 x 9 x 7 image, C = 48 (one partial 64-channel chunk), K = 80 (partial k block)
    xq, wq, s_x, s_w = small_layer(3, 9, 7, 48, 80, seed=50 + m)
    run_fused(xq, wq, s_x, s_w, m=m, base=base, bits_hadamard=bits_hadamard, out_type="i8")
    run_fused(xq, wq, s_x, s_w, m=m, base=base, bits_hadamard=bits_hadamard, out_type="f32",
              relu=True)


def test_fused_equals_split_path_bit_for_bit():
    xq, wq, s_x, s_w = small_layer(5, 8, 8, 128, 64, seed=60)       # two channel chunks
    got, sc = run_fused(xq, wq, s_x, s_w, m=4, base="legendre", out_type="i8", relu=True)
    split = gpu_layer(xq, wq, sc, m=4, base="legendre", out_type="i8", relu=True, whole=True)
    assert np.array_equal(split["y"], got["y"])


@pytest.mark.parametrize("name", ["cfg1_f2_canonical", "cfg1_f2_legendre", "cfg2_f4_c64",
                                  "cfg3_f4_c128_h9", "cfg4a_f4_c256"])
def test_fused_benchmark_configurations(name):
    wl = si.WORKLOADS[name]
    L = si.make_layer(wl)
    run_fused(L["xq"], L["wq"], L["s_x"], L["s_w"], m=wl.m, base=wl.base,
              bits_hadamard=wl.bits_hadamard, out_type="i8")
    run_fused(L["xq"], L["wq"], L["s_x"], L["s_w"], m=wl.m, base=wl.base,
              bits_hadamard=wl.bits_hadamard, out_type="f32")


def test_fused_rejects_what_it_does_not_cover():
    import paper_2004_11077_amd as wn
    for kw in (dict(bits_hadamard=32), dict(bits_in=32),
               dict(base=wn.BASE_CANONICAL, out_type=wn.OUT_I32)):
        with pytest.raises(wn.WinoError) as e:
            import torch
            d = wn.ConvDesc(1, 8, 8, 16, 16, fused=1, **kw)
            buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
            wn.wino_conv2d(d, buf, buf, buf, wn.Scales.from_dict({}), buf)
        assert e.value.code == -2


def test_auto_mode_picks_a_variant_and_matches_the_split_path():
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    for (C, K) in [(64, 64), (128, 64)]:           # fused is chosen for the first, split for the second
        xq, wq, s_x, s_w = small_layer(4, 8, 8, C, K, seed=95)
        ora, sc = oracle_layer(xq, wq, s_x, s_w, m=4, base="legendre", out_type="i8")
        desc = wn.ConvDesc(4, 8, 8, C, K, m=4, out_type=wn.OUT_I8, fused=wn.FUSED_AUTO)
        x = torch.from_numpy(xq).to(dev)
        w = torch.from_numpy(wq).to(dev)
        y = torch.full((4, 8, 8, K), 77, dtype=torch.int8, device=dev)
        ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        wn.wino_conv2d(desc, x, w, y, wn.Scales.from_dict(sc), ws)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().astype(np.int64), ora["y"])
    with pytest.raises(wn.WinoError):
        wn.wino_workspace_bytes(wn.ConvDesc(1, 8, 8, 16, 16, fused=7)) and None
        d = wn.ConvDesc(1, 8, 8, 16, 16, fused=7)
        buf = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
        wn.wino_conv2d(d, buf, buf, buf, wn.Scales.from_dict({}), buf)
