"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Bar: int8 transformed tensors (V, U), contraction results (int32, and the
8 / 9-bit codes) and integer outputs bit-exact; dequantised fp32 outputs within
max abs error 1e-5 * max|y_oracle|.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import quantised as oq
from helpers import assert_layer_parity, gpu_layer, oracle_layer, small_layer

pytestmark = pytest.mark.gpu


def run_case(xq, wq, s_x, s_w, whole=False, **kw):
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got = gpu_layer(xq, wq, sc, whole=whole, **kw)
    assert_layer_parity(ora, got, kw.get("out_type", "f32"))
    return ora, got, sc


@pytest.mark.parametrize("name", ["cfg1_f2_canonical", "cfg1_f2_legendre"])
def test_cfg1(name):
    wl = si.WORKLOADS[name]
    L = si.make_layer(wl)
    run_case(L["xq"], L["wq"], L["s_x"], L["s_w"], m=wl.m, base=wl.base)
    run_case(L["xq"], L["wq"], L["s_x"], L["s_w"], m=wl.m, base=wl.base, whole=True)


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("base", ["canonical", "legendre"])
@pytest.mark.parametrize("bits_hadamard", [8, 9, 32])
def test_small_ragged_all_variants(m, base, bits_hadamard):
    # several tiles per image, ragged bottom/right edge, tile and channel
    # counts that are not multiples of the kernels' block sizes
    xq, wq, s_x, s_w = small_layer(3, 9, 7, 48, 80, seed=20 + m)
    run_case(xq, wq, s_x, s_w, m=m, base=base, bits_hadamard=bits_hadamard)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_int8_output_with_relu_and_whole_layer_call(m):
    xq, wq, s_x, s_w = small_layer(2, 8, 8, 32, 32, seed=31)
    for base in ("canonical", "legendre"):
        run_case(xq, wq, s_x, s_w, m=m, base=base, out_type="i8", relu=True, whole=True)
        run_case(xq, wq, s_x, s_w, m=m, base=base, out_type="f32", relu=True)


@pytest.mark.parametrize("m", [2, 4])
def test_int32_output_canonical(m):
    xq, wq, s_x, s_w = small_layer(2, 8, 8, 32, 32, seed=32)
    run_case(xq, wq, s_x, s_w, m=m, base="canonical", out_type="i32")
    run_case(xq, wq, s_x, s_w, m=m, base="canonical", out_type="i32", bits_hadamard=32)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_legendre_without_inner_casts_equals_canonical_on_gpu(m):
    xq, wq, s_x, s_w = small_layer(2, 8, 8, 32, 32, seed=33)
    ora, got, sc = run_case(xq, wq, s_x, s_w, m=m, base="legendre", inner_quant=False)
    can = gpu_layer(xq, wq, sc, m=m, base="canonical")
    for key in ("V", "U", "M", "y"):
        assert np.array_equal(can[key], got[key])


def test_degenerate_shapes():
    # one pixel, one tile; and an image smaller than a tile with m = 6
    for (N, H, W, m) in [(1, 1, 1, 4), (2, 4, 4, 6), (1, 2, 3, 2)]:
        xq, wq, s_x, s_w = small_layer(N, H, W, 16, 16, seed=34)
        run_case(xq, wq, s_x, s_w, m=m, base="legendre")


def test_saturating_scales_clamp_symmetrically():
    xq, wq, s_x, s_w = small_layer(1, 8, 8, 16, 16, seed=35)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, m=4, base="legendre")
    tight = {k: (np.float32(v * 0.25) if k in ("s_u", "s_v", "s_m", "s_x1") else v)
             for k, v in sc.items()}
    ora2, _ = oq.run_layer(xq, wq, s_x, s_w, oq.LayerConfig(m=4), scales=tight)
    got = gpu_layer(xq, wq, tight, m=4, base="legendre")
    assert_layer_parity(ora2, got)
    assert got["U"].min() == -127 and got["U"].max() == 127


FULL = ["cfg2_f4_c64", "cfg3_f4_c128_h9", "cfg4a_f4_c256", "cfg4b_f4_c512", "cfg4a_f6_c256",
        "cfg4b_f6_c512"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_configurations(name):
    """The benchmark shapes, whole-layer call, every element compared."""
    wl = si.WORKLOADS[name]
    L = si.make_layer(wl)
    run_case(L["xq"], L["wq"], L["s_x"], L["s_w"], whole=True, m=wl.m, base=wl.base,
             bits_hadamard=wl.bits_hadamard)


@pytest.mark.parametrize("m,base,shape,bh,out_type,relu", [
    (2, "canonical", (2, 5, 7, 256, 256), 8, "i8", True),
    (4, "legendre", (1, 9, 6, 512, 256), 9, "f32", False),
    (4, "canonical", (2, 6, 6, 256, 512), 8, "i32", True),
    (6, "legendre", (1, 7, 7, 256, 512), 8, "i8", False),
])
def test_channel_counts_that_are_multiples_of_256(m, base, shape, bh, out_type, relu):
    """Such layers take the transform kernels whose tile arithmetic is block-uniform;
    ragged images, every output type, split and whole-layer calls."""
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=90 + m)
    for whole in (False, True):
        run_case(xq, wq, s_x, s_w, whole=whole, m=m, base=base, bits_hadamard=bh,
                 out_type=out_type, relu=relu)


@pytest.mark.parametrize("m,shape", [(4, (1, 113, 57, 32, 16)), (6, (1, 64, 200, 16, 32)),
                                     (2, (2, 75, 75, 16, 16))])
def test_large_ragged_images(m, shape):
    """Many tiles per image, edges that are not multiples of m in either direction."""
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=130 + m)
    run_case(xq, wq, s_x, s_w, whole=True, m=m, base="legendre", out_type="i8", relu=True)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_operand_transforms_in_one_launch_equal_the_two_calls(m):
    import torch
    import paper_2004_11077_amd as wn
    xq, wq, s_x, s_w = small_layer(3, 9, 7, 48, 80, seed=70 + m)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, m=m)
    dev = torch.device("cuda:0")
    desc = wn.ConvDesc(3, 9, 7, 48, 80, m=m)
    n2, T = desc.n ** 2, desc.tiles
    x = torch.from_numpy(xq).to(dev)
    w = torch.from_numpy(wq).to(dev)
    U = torch.full((n2, T, 48), 77, dtype=torch.int8, device=dev)
    V = torch.full((n2, 80, 48), 77, dtype=torch.int8, device=dev)
    wn.wino_transform_operands(desc, x, U, w, V, wn.Scales.from_dict(sc))
    torch.cuda.synchronize()
    assert np.array_equal(U.cpu().numpy().astype(np.int64), ora["U"])
    assert np.array_equal(V.cpu().numpy().astype(np.int64), ora["V"])


def test_empty_batch_is_a_no_op():
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    desc = wn.ConvDesc(0, 8, 8, 16, 16, m=4)
    e8 = torch.empty(0, dtype=torch.int8, device=dev)
    y = torch.empty((0, 8, 8, 16), dtype=torch.float32, device=dev)
    w = torch.zeros((16, 16, 3, 3), dtype=torch.int8, device=dev)
    ws = torch.empty(max(256, wn.wino_workspace_bytes(desc)), dtype=torch.uint8, device=dev)
    sc = wn.Scales.from_dict({})
    wn.wino_conv2d(desc, e8, w, y, sc, ws)
    wn.wino_input_transform(desc, e8, e8, sc)
    wn.wino_contract(desc, e8, ws, e8, sc)
    wn.wino_output_transform(desc, e8, y, sc)
    torch.cuda.synchronize()


def test_largest_exact_contraction_result():
    """bits_hadamard = 32 at the channel limit (C = 1040): saturated codes give
    127 * 127 * 1040 = 16 774 160 < 2^24, the largest value that the output bracket
    still converts to fp32 exactly."""
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K, m = 1, 4, 8, 1040, 16, 4
    desc = wn.ConvDesc(N, H, W, C, K, m=m, base=wn.BASE_CANONICAL, bits_hadamard=32)
    n2, T = 36, desc.tiles
    rng = np.random.default_rng(5)
    sign_u = rng.choice([-127, 127], size=(n2, T, 1)).astype(np.int8)
    sign_v = rng.choice([-127, 127], size=(n2, K, 1)).astype(np.int8)
    Uq = np.broadcast_to(sign_u, (n2, T, C)).copy()
    Vq = np.broadcast_to(sign_v, (n2, K, C)).copy()
    sc = {"s_x": 1.0, "s_w": 1.0, "s_u": 0.5, "s_v": 0.25}
    cfg = oq.LayerConfig(m=m, base="canonical", bits_hadamard=32)
    out = {}
    Mq, s_m = oq.contraction(Uq.astype(np.int64), Vq.astype(np.int64), cfg, dict(sc), out)
    assert np.abs(Mq).max() == 127 * 127 * 1040
    y_ref = oq.output_transform(Mq, s_m, (N, H, W), cfg, oq.StageMatrices(cfg), dict(sc), out)
    U = torch.from_numpy(Uq).to(dev)
    V = torch.from_numpy(Vq).to(dev)
    M = torch.zeros((n2, T, K), dtype=torch.int32, device=dev)
    y = torch.zeros((N, H, W, K), dtype=torch.float32, device=dev)
    gsc = wn.Scales.from_dict(sc)
    wn.wino_contract(desc, U, V, M, gsc)
    wn.wino_output_transform(desc, M, y, gsc)
    torch.cuda.synchronize()
    assert np.array_equal(M.cpu().numpy().astype(np.int64), Mq)
    err = np.abs(y.cpu().numpy().astype(np.float64) - y_ref).max()
    assert err <= 1e-5 * np.abs(y_ref).max()


@pytest.mark.parametrize("bits_hadamard", [8, 9, 32])
def test_no_input_channels_gives_zero_output(bits_hadamard):
    """C = 0 with tiles and output channels present: an empty channel sum.  The contraction
    stage must not read U or V (there is nothing to read) and every M and y is zero; split
    calls and the whole-layer call in all three fused modes."""
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K, m = 2, 9, 7, 0, 32, 4
    mdt = {8: torch.int8, 9: torch.int16, 32: torch.int32}[bits_hadamard]
    sc = wn.Scales.from_dict({k: 0.5 for k in ("s_x", "s_x1", "s_u", "s_w", "s_w1", "s_v", "s_m",
                                               "s_m1", "s_y")})
    x = torch.empty((N, H, W, 0), dtype=torch.int8, device=dev)
    w = torch.empty((K, 0, 3, 3), dtype=torch.int8, device=dev)
    desc = wn.ConvDesc(N, H, W, C, K, m=m, bits_hadamard=bits_hadamard)
    n2, T = desc.n ** 2, desc.tiles
    M = torch.full((n2, T, K), 77, dtype=mdt, device=dev)
    y = torch.full((N, H, W, K), 7.0, dtype=torch.float32, device=dev)
    wn.wino_contract(desc, None, None, M, sc)    # U and V are empty: null pointers are accepted
    wn.wino_output_transform(desc, M, y, sc)
    torch.cuda.synchronize()
    assert int(M.abs().max()) == 0 and float(y.abs().max()) == 0.0
    modes = [wn.FUSED_OFF, wn.FUSED_AUTO] + ([wn.FUSED_ON] if bits_hadamard != 32 else [])
    for mode in modes:
        d2 = wn.ConvDesc(N, H, W, C, K, m=m, bits_hadamard=bits_hadamard, fused=mode)
        ws = torch.full((wn.wino_workspace_bytes(d2),), 77, dtype=torch.uint8, device=dev)
        y2 = torch.full((N, H, W, K), 7.0, dtype=torch.float32, device=dev)
        wn.wino_conv2d(d2, x, w, y2, sc, ws)
        torch.cuda.synchronize()
        assert float(y2.abs().max()) == 0.0, mode
