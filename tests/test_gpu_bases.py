"""GPU parity of the layer in the other polynomial bases Section 4.1 names: the two-bracket
form of eq. 2 / eq. 4 with P built from the monic Chebyshev and the monic Hermite polynomials,
against the oracle's LayerConfig.base.

Bar as for the Legendre base: V, U, M and integer outputs bit-exact, fp32 outputs within
1e-5 * max|y_oracle|; stage calls and the whole-layer call (one kernel per stage).
"""
import numpy as np
import pytest

from helpers import assert_layer_parity, gpu_layer, oracle_layer, small_layer

pytestmark = pytest.mark.gpu

BASES = ["chebyshev", "hermite"]


@pytest.mark.parametrize("base", BASES)
@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("bits_hadamard", [8, 9, 32])
def test_stage_calls_small_ragged(base, m, bits_hadamard):
    # several tiles per image, ragged edges, channel counts that are not multiples of a block
    xq, wq, s_x, s_w = small_layer(3, 9, 7, 48, 80, seed=820 + m)
    kw = dict(m=m, base=base, bits_hadamard=bits_hadamard)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got = gpu_layer(xq, wq, sc, **kw)
    assert_layer_parity(ora, got)


@pytest.mark.parametrize("base", BASES)
@pytest.mark.parametrize("m", [2, 4, 6])
def test_whole_layer_int8_output_with_relu(base, m):
    xq, wq, s_x, s_w = small_layer(2, 11, 8, 256, 32, seed=830 + m)     # C a multiple of 256
    kw = dict(m=m, base=base, out_type="i8", relu=True)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    got = gpu_layer(xq, wq, sc, whole=True, **kw)
    assert_layer_parity(ora, got, "i8")
    assert got["y"].min() >= 0


@pytest.mark.parametrize("base", BASES)
@pytest.mark.parametrize("m", [2, 4, 6])
def test_without_inner_casts_the_base_drops_out(base, m):
    """inner_quant = 0 multiplies each bracket pair out: the layer must equal the canonical one
    bit for bit, whatever P is."""
    xq, wq, s_x, s_w = small_layer(2, 8, 8, 32, 32, seed=840 + m)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, m=m, base=base, inner_quant=False)
    got = gpu_layer(xq, wq, sc, m=m, base=base, inner_quant=False)
    assert_layer_parity(ora, got)
    can = gpu_layer(xq, wq, sc, m=m, base="canonical")
    for key in ("V", "U", "M", "y"):
        assert np.array_equal(can[key], got[key])


def test_benchmark_shape_in_both_bases():
    import synth_inputs as si
    wl = si.WORKLOADS["cfg4a_f4_c256"]
    x, w = si.make_real(32, wl.H, wl.W, wl.C, wl.K, wl.seed, wl.outliers)
    xq, s_x = si.cast_int8(x)
    wq, s_w = si.cast_int8(w)
    for base in BASES:
        ora, sc = oracle_layer(xq, wq, s_x, s_w, m=4, base=base)
        got = gpu_layer(xq, wq, sc, m=4, base=base, whole=True)
        assert_layer_parity(ora, got)


def test_variants_that_are_not_built_for_these_bases_say_so():
    import torch
    import paper_2004_11077_amd as wn
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    s = wn.Scales.from_dict({})
    for base in (wn.BASE_CHEBYSHEV, wn.BASE_HERMITE):
        d = wn.ConvDesc(1, 8, 8, 16, 16, base=base, fused=wn.FUSED_ON)
        with pytest.raises(wn.WinoError) as e:
            wn.wino_conv2d(d, buf, buf, buf, s, buf)
        assert e.value.code == -2
        with pytest.raises(wn.WinoError) as e:
            wn.wino_contract_output(wn.ConvDesc(1, 8, 8, 16, 16, base=base), buf, buf, buf, s)
        assert e.value.code == -2
        with pytest.raises(wn.WinoError) as e:
            wn.wino_calibrate(wn.ConvDesc(1, 8, 8, 16, 16, base=base), buf, buf, None, 1.0, 1.0, buf)
        assert e.value.code == -2
