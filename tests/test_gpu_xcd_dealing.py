"""GPU parity on layers where the transforms deal their work groups to XCDs in units (an
image, a 32-tile block, an eighth of the tiles) and the dealt range ends before the last
work group: every tile must still be transformed exactly once, whatever the order."""
import pytest

from helpers import assert_layer_parity, gpu_layer, oracle_layer, small_layer

pytestmark = pytest.mark.gpu

CASES = [
    # an eighth of the tiles per XCD through all three stage kernels (T = 512 = 8 x 64)
    dict(N=128, H=8, W=8, C=256, K=256, m=4, base="legendre", bits_hadamard=8, out_type="f32"),
    # fragment order: 11 blocks of 32 tiles and 8 tiles more, 8 blocks dealt
    dict(N=40, H=10, W=10, C=128, K=64, m=4, base="legendre", bits_hadamard=8, out_type="i8"),
    # fragment order: 21 blocks and 12 tiles more, 16 blocks dealt; 9-bit codes
    dict(N=19, H=12, W=12, C=256, K=256, m=2, base="canonical", bits_hadamard=9, out_type="f32"),
    # rows, one image per unit: 9 images, 8 dealt
    dict(N=9, H=16, W=16, C=256, K=256, m=4, base="legendre", bits_hadamard=8, out_type="i8"),
    # F(6,3): 64 points, tiles that reach past the image
    dict(N=33, H=8, W=8, C=256, K=256, m=6, base="legendre", bits_hadamard=8, out_type="f32"),
]


@pytest.mark.parametrize("c", CASES, ids=lambda c: "N%(N)d_%(H)dx%(W)d_C%(C)d_K%(K)d_F%(m)d_h%(bits_hadamard)d" % c)
def test_dealt_layers_match_the_oracle(c):
    xq, wq, s_x, s_w = small_layer(c["N"], c["H"], c["W"], c["C"], c["K"], seed=900 + c["N"])
    kw = dict(m=c["m"], base=c["base"], bits_hadamard=c["bits_hadamard"], out_type=c["out_type"],
              relu=True)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
    assert_layer_parity(ora, gpu_layer(xq, wq, sc, **kw), c["out_type"])              # stage calls
    assert_layer_parity(ora, gpu_layer(xq, wq, sc, whole=True, **kw), c["out_type"])  # wino_conv2d
    assert_layer_parity(ora, gpu_layer(xq, wq, sc, fused=True, **kw), c["out_type"])  # fused = ON
