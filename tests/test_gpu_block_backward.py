"""Forward and backward pass of a residual block of two Winograd layers through the library:

    y1 = Q8(ReLU(conv1(x)))      int8 output of layer 1 = int8 input of layer 2
    out = conv2(y1) + x_real     fp32, identity skip (C = K)

Backward, with straight-through casts: layer 2 gives the gradient with respect to its real
input s_y1 * y1; it passes the cast unchanged and the ReLU where the code is positive, becomes
the output gradient of layer 1, and the skip adds d(out) to dx.  The glue between the layers
(mask, additions) is the caller's; each layer's gradients are checked against the oracle chain.
"""
import numpy as np
import pytest

from helpers import gpu_layer, oracle_layer, small_layer
from oracle import backward as bw
import synth_inputs as si

pytestmark = pytest.mark.gpu


def layer_backward_gpu(dy, Uq, Vq, sc, shape, m):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K = shape
    desc = wn.ConvDesc(N, H, W, C, K, m=m)
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(dev)
    dx = torch.empty((N, H, W, C), dtype=torch.float32, device=dev)
    dw = torch.empty((K, C, 3, 3), dtype=torch.float32, device=dev)
    ws = torch.empty(wn.wino_backward_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    wn.wino_backward(desc, t(dy, np.float32), t(Uq, np.int8), t(Vq, np.int8),
                     wn.Scales.from_dict({"s_u": float(sc["s_u"]), "s_v": float(sc["s_v"])}), dx, dw, ws)
    torch.cuda.synchronize()
    return dx.cpu().numpy(), dw.cpu().numpy()


@pytest.mark.parametrize("m,base", [(4, "legendre"), (2, "canonical")])
def test_residual_block_forward_and_backward(m, base):
    N, H, W, C = 4, 8, 8, 64
    shape = (N, H, W, C, C)
    xq, w1q, s_x, s_w1 = small_layer(N, H, W, C, C, seed=41)
    _, w2 = si.make_real(1, 1, 1, C, C, seed=42)
    w2q, s_w2 = si.cast_int8(w2)
    d_out = np.random.default_rng(43).standard_normal((N, H, W, C)).astype(np.float32)

    # forward: oracle and library, layer by layer (integer tensors bit-exact)
    kw1 = dict(m=m, base=base, out_type="i8", relu=True)
    kw2 = dict(m=m, base=base, out_type="f32")
    o1, sc1 = oracle_layer(xq, w1q, s_x, s_w1, **kw1)
    g1 = gpu_layer(xq, w1q, sc1, **kw1)
    assert np.array_equal(g1["y"].astype(np.int64), o1["y"])
    y1q, s_y1 = g1["y"], sc1["s_y"]
    o2, sc2 = oracle_layer(y1q, w2q, s_y1, s_w2, **kw2)
    g2 = gpu_layer(y1q, w2q, sc2, **kw2)
    for key in ("U", "V"):
        assert np.array_equal(g1[key].astype(np.int64), o1[key])
        assert np.array_equal(g2[key].astype(np.int64), o2[key])

    # backward: oracle chain in fp64
    r2 = bw.backward_layer(d_out.astype(np.float64), bw.dequantise(o2["U"], sc2["s_u"]),
                           bw.dequantise(o2["V"], sc2["s_v"]), xq.shape, m)
    mask = (o1["y"] > 0)
    r1 = bw.backward_layer(r2["dx"] * mask, bw.dequantise(o1["U"], sc1["s_u"]),
                           bw.dequantise(o1["V"], sc1["s_v"]), xq.shape, m)
    ref_dx = r1["dx"] + d_out

    # backward: library, the glue in numpy on the host
    dx2, dw2 = layer_backward_gpu(d_out, g2["U"], g2["V"], sc2, shape, m)
    dy1 = dx2 * (g1["y"] > 0)
    dx1, dw1 = layer_backward_gpu(dy1, g1["U"], g1["V"], sc1, shape, m)
    dx = dx1 + d_out

    for name, got, ref in (("dw2", dw2, r2["dw"]), ("dw1", dw1, r1["dw"]), ("dx", dx, ref_dx)):
        err, top = float(np.abs(got - ref).max()), float(np.abs(ref).max())
        assert err <= 2e-5 * top, "%s: %g > %g" % (name, err, 2e-5 * top)   # two chained fp32 passes
