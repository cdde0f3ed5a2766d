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
    if c["m"] != 6 and c["bits_hadamard"] != 32:
        assert_layer_parity(ora, gpu_layer(xq, wq, sc, fused=True, **kw), c["out_type"])
