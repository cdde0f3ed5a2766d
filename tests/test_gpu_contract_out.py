"""GPU parity of the kernel that runs the Hadamard stage and the output bracket of
eq. 3 / eq. 4 in one launch (the cast contraction result M stays in on-chip memory).

Bar: int8 outputs bit-exact against the oracle (an int8 y that matches bit for bit also pins
the M codes it was computed from, since every one of them feeds the integer brackets); fp32
outputs within 1e-5 * max|y_oracle|, and bit-identical to what wino_contract followed by
wino_output_transform give on the same U and V (the arithmetic is the same).  The operands
are given in rows and in fragment order (the
fragment-order tensors must hold exactly the row-order codes, zeros in V's channel padding);
shapes are chosen so that tiles, output channels and input channels all end in partial blocks
/ chunks.
"""
import numpy as np
import pytest

import synth_inputs as si
from helpers import assert_layer_parity, gpu_layer, oracle_layer, small_layer

pytestmark = pytest.mark.gpu


def stage_call(xq, wq, sc, frag=False, **kw):
    """U and V from the stage calls (rows, or fragment order when ``frag``), then y from
    wino_contract_output and, for comparison, from wino_contract + wino_output_transform."""
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = xq.shape
    K = wq.shape[0]
    out_type = kw.get("out_type", "f32")
    bh = kw.get("bits_hadamard", 8)
    common = dict(m=kw["m"],
                  base=wn.BASE_LEGENDRE if kw["base"] == "legendre" else wn.BASE_CANONICAL,
                  bits_hadamard=bh, inner_quant=int(kw.get("inner_quant", True)),
                  out_type=wn.OUT_I8 if out_type == "i8" else wn.OUT_F32,
                  relu=int(kw.get("relu", False)))
    desc = wn.ConvDesc(N, H, W, C, K, **common)
    n2, T = desc.n ** 2, desc.tiles
    s = wn.Scales.from_dict(sc)
    x = torch.from_numpy(np.ascontiguousarray(xq, dtype=np.int8)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq, dtype=np.int8)).to(dev)
    ydt = torch.int8 if out_type == "i8" else torch.float32
    U = torch.empty((n2, T, C), dtype=torch.int8, device=dev)
    V = torch.empty((n2, K, C), dtype=torch.int8, device=dev)
    M = torch.empty((n2, T, K), dtype=torch.int8 if bh == 8 else torch.int16, device=dev)
    y = torch.full((N, H, W, K), 77, dtype=ydt, device=dev)
    y2 = torch.full((N, H, W, K), 55, dtype=ydt, device=dev)
    wn.wino_transform_operands(desc, x, U, w, V, s)
    Uc, Vc, dc = U, V, desc
    if frag:
        dc = wn.ConvDesc(N, H, W, C, K, operand_layout=wn.LAYOUT_FRAGMENTS, **common)
        vb, ub = wn.wino_operand_bytes(dc)
        Uc = torch.full((ub,), 77, dtype=torch.int8, device=dev)
        Vc = torch.full((vb,), 77, dtype=torch.int8, device=dev)
        wn.wino_transform_operands(dc, x, Uc, w, Vc, s)
    wn.wino_contract_output(dc, Uc, Vc, y, s)
    wn.wino_contract(desc, U, V, M, s)
    wn.wino_output_transform(desc, M, y2, s)
    torch.cuda.synchronize()
    if frag:
        # the same codes, in fragment order; channels of V past C are zeros
        Un = wn.defragment(Uc.cpu().numpy(), n2, T, C)
        Vn = wn.defragment(Vc.cpu().numpy(), n2, K, C)
        assert np.array_equal(Un, U.cpu().numpy()) and np.array_equal(Vn, V.cpu().numpy())
        if C % 64:
            pad = Vc.cpu().numpy().reshape(n2, K // 16, -1, 4, 16, 16)[:, :, -1, (C % 64) // 16:]
            assert not pad.any()
    return {"U": U.cpu().numpy(), "V": V.cpu().numpy(), "y": y.cpu().numpy()}, y2.cpu().numpy()


CASES = [
    # m, base, (N, H, W, C, K), bits_hadamard, out_type, relu, per_point
    (4, "legendre", (3, 9, 7, 48, 80), 8, "i8", False, False),
    (4, "legendre", (3, 9, 7, 48, 80), 9, "f32", True, False),
    (4, "canonical", (2, 11, 6, 80, 48), 8, "f32", False, False),
    (4, "canonical", (5, 8, 8, 272, 112), 9, "i8", True, False),
    (4, "legendre", (7, 8, 8, 256, 64), 8, "i8", True, True),
    (4, "canonical", (2, 12, 12, 144, 96), 9, "f32", False, True),
    (2, "legendre", (3, 9, 7, 48, 80), 8, "i8", True, False),
    (2, "canonical", (9, 8, 8, 64, 16), 9, "f32", False, True),
    (6, "legendre", (2, 13, 11, 48, 80), 8, "i8", False, False),
    (6, "canonical", (3, 12, 12, 128, 48), 9, "f32", True, False),
    (6, "legendre", (2, 7, 8, 32, 16), 9, "i8", True, True),
]


@pytest.mark.parametrize("frag", [False, True])
@pytest.mark.parametrize("m,base,shape,bh,out_type,relu,pp", CASES)
def test_stage_call_matches_the_oracle_and_the_two_stage_calls(m, base, shape, bh, out_type, relu,
                                                               pp, frag):
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=700 + m + C, outliers=0.01 if pp else 0.0)
    kw = dict(m=m, base=base, bits_hadamard=bh, out_type=out_type, relu=relu, per_point=pp)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got, y_two = stage_call(xq, wq, sc, frag=frag, **kw)
    assert_layer_parity(ora, got, out_type)
    assert np.array_equal(got["y"], y_two)


def test_legendre_without_inner_casts():
    xq, wq, s_x, s_w = small_layer(2, 8, 8, 32, 32, seed=733)
    kw = dict(m=4, base="legendre", inner_quant=False, out_type="i8")
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got, y_two = stage_call(xq, wq, sc, **kw)
    assert_layer_parity(ora, got, "i8")


def whole_layer(xq, wq, sc, mode, pretransformed=False, **kw):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = xq.shape
    K = wq.shape[0]
    out_type = kw.get("out_type", "f32")
    common = dict(m=kw["m"], base=wn.BASE_LEGENDRE if kw["base"] == "legendre" else wn.BASE_CANONICAL,
                  bits_hadamard=kw.get("bits_hadamard", 8),
                  out_type=wn.OUT_I8 if out_type == "i8" else wn.OUT_F32,
                  relu=int(kw.get("relu", False)))
    s = wn.Scales.from_dict(sc)
    x = torch.from_numpy(np.ascontiguousarray(xq, dtype=np.int8)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq, dtype=np.int8)).to(dev)
    y = torch.full((N, H, W, K), 77, dtype=torch.int8 if out_type == "i8" else torch.float32,
                   device=dev)
    second, layout = w, wn.LAYOUT_ROWS
    if pretransformed:
        layout = (wn.LAYOUT_FRAGMENTS if mode == wn.FUSED_ON else
                  wn.wino_preferred_operand_layout(wn.ConvDesc(N, H, W, C, K, **common)))
        vdesc = wn.ConvDesc(N, H, W, C, K, operand_layout=layout, **common)
        second = torch.empty((wn.wino_operand_bytes(vdesc)[0],), dtype=torch.int8, device=dev)
        wn.wino_weight_transform(vdesc, w, second, s)
    desc = wn.ConvDesc(N, H, W, C, K, fused=mode, weights_pretransformed=int(pretransformed),
                       operand_layout=layout, **common)
    if mode == wn.FUSED_ON:
        single = C <= 64 and kw["m"] in (2, 4)       # narrow layers: everything in one kernel
        assert ("fused_layer" if single else "contraction_output") in wn.wino_conv2d_launches(desc)
    ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    wn.wino_conv2d(desc, x, second, y, s, ws)
    torch.cuda.synchronize()
    return {"y": y.cpu().numpy()}


FULL = ["cfg3_f4_c128_h9", "cfg4a_f4_c256", "cfg4b_f4_c512", "cfg4a_f6_c256", "cfg4b_f6_c512"]


@pytest.mark.parametrize("name", FULL)
def test_whole_layer_call_on_the_benchmark_configurations(name):
    """fused = AUTO and ON at the full benchmark sizes: int8 and fp32 output, per-tensor and
    per-point scales, filters given raw or transformed beforehand."""
    import paper_2004_11077_amd as wn
    wl = si.WORKLOADS[name]
    L = si.make_layer(wl)
    for out_type, pp, mode, pre in [("i8", False, wn.FUSED_AUTO, False),
                                    ("f32", False, wn.FUSED_ON, True),
                                    ("i8", True, wn.FUSED_AUTO, True)]:
        kw = dict(m=wl.m, base=wl.base, bits_hadamard=wl.bits_hadamard, out_type=out_type,
                  per_point=pp)
        ora, sc = oracle_layer(L["xq"], L["wq"], L["s_x"], L["s_w"], **kw)
        kw.pop("per_point")
        got = whole_layer(L["xq"], L["wq"], sc, mode, pretransformed=pre, **kw)
        assert_layer_parity(ora, got, out_type)


def test_many_tile_blocks_per_compute_unit():
    """Several rounds of work groups per compute unit (4096 tiles), whole-layer call against
    the oracle."""
    import paper_2004_11077_amd as wn
    xq, wq, s_x, s_w = small_layer(64, 32, 32, 128, 128, seed=741)       # T = 4096
    kw = dict(m=4, base="legendre", out_type="i8", relu=True)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got = whole_layer(xq, wq, sc, wn.FUSED_ON, **kw)
    assert_layer_parity(ora, got, "i8")
