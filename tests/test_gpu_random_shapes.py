"""GPU parity on seeded random shapes and option combinations (split, whole-layer
and fused calls), to catch corner cases of tiling, channel tails and block edges."""
import numpy as np
import pytest

from helpers import assert_layer_parity, gpu_layer, oracle_layer, small_layer

pytestmark = pytest.mark.gpu


def cases():
    rng = np.random.default_rng(2024)
    out = []
    for i in range(24):
        m = int(rng.choice([2, 4, 6]))
        out.append(dict(
            N=int(rng.integers(1, 4)), H=int(rng.integers(1, 14)), W=int(rng.integers(1, 14)),
            C=int(rng.choice([16, 32, 48, 64, 80, 144, 272])),
            K=int(rng.choice([16, 32, 48, 64, 80, 144])),
            m=m, base=str(rng.choice(["canonical", "legendre"])),
            bits_hadamard=int(rng.choice([8, 9, 32])),
            out_type=str(rng.choice(["f32", "i8"])), relu=bool(rng.integers(0, 2)), seed=100 + i))
    return out


@pytest.mark.parametrize("c", cases(), ids=lambda c: "N%(N)d_%(H)dx%(W)d_C%(C)d_K%(K)d_F%(m)d_%(base)s_h%(bits_hadamard)d_%(out_type)s" % c)
def test_random_case(c):
    xq, wq, s_x, s_w = small_layer(c["N"], c["H"], c["W"], c["C"], c["K"], c["seed"])
    kw = dict(m=c["m"], base=c["base"], bits_hadamard=c["bits_hadamard"], out_type=c["out_type"],
              relu=c["relu"])
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    assert_layer_parity(ora, gpu_layer(xq, wq, sc, **kw), c["out_type"])
    assert_layer_parity(ora, gpu_layer(xq, wq, sc, whole=True, **kw), c["out_type"])
    if c["bits_hadamard"] != 32:
        # fused = ON: the single kernel (C <= 64, F(2,3) / F(4,3)) or contraction + output in one
        assert_layer_parity(ora, gpu_layer(xq, wq, sc, fused=True, **kw), c["out_type"])


def option_cases():
    rng = np.random.default_rng(4048)
    out = []
    for i in range(20):
        out.append(dict(
            N=int(rng.integers(1, 6)), H=int(rng.integers(1, 18)), W=int(rng.integers(1, 18)),
            C=int(rng.choice([16, 48, 64, 96, 128, 208, 256])),
            K=int(rng.choice([16, 32, 64, 96, 128, 160])),
            m=int(rng.choice([2, 4, 6])), base=str(rng.choice(["canonical", "legendre"])),
            bits_hadamard=int(rng.choice([8, 9])), out_type=str(rng.choice(["f32", "i8"])),
            relu=bool(rng.integers(0, 2)), per_point=bool(rng.integers(0, 2)),
            mode=str(rng.choice(["auto", "on"])), pre=bool(rng.integers(0, 2)), seed=300 + i))
    return out


@pytest.mark.parametrize("c", option_cases(), ids=lambda c: "N%(N)d_%(H)dx%(W)d_C%(C)d_K%(K)d_F%(m)d_%(base)s_h%(bits_hadamard)d_%(out_type)s_pp%(per_point)d_%(mode)s_pre%(pre)d" % c)
def test_random_case_whole_layer_options(c):
    """Whole-layer calls with per-point scales, fused = AUTO / ON, and filters given raw or
    transformed beforehand in the layout the library prefers (ON: fragment order)."""
    import paper_2004_11077_amd as wn
    from test_gpu_contract_out import whole_layer
    xq, wq, s_x, s_w = small_layer(c["N"], c["H"], c["W"], c["C"], c["K"], c["seed"],
                                   outliers=0.01 if c["per_point"] else 0.0)
    kw = dict(m=c["m"], base=c["base"], bits_hadamard=c["bits_hadamard"], out_type=c["out_type"],
              relu=c["relu"])
    ora, sc = oracle_layer(xq, wq, s_x, s_w, per_point=c["per_point"], **kw)
    mode = wn.FUSED_ON if c["mode"] == "on" else wn.FUSED_AUTO
    pre = c["pre"]
    if mode == wn.FUSED_ON and pre and c["C"] <= 64 and c["m"] != 6:
        pre = False          # the single kernel reads V in rows; whole_layer hands ON fragments
    got = whole_layer(xq, wq, sc, mode, pretransformed=pre, **kw)
    assert_layer_parity(ora, got, c["out_type"])
