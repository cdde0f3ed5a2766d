"""GPU parity on the ResNet18-style 3x3 stack (the fifth benchmark configuration).

The 14 enumerated stride-1 layers (stem 3->64 at 32x32, 4 x 64 at 32x32,
3 x 128 at 16x16, 3 x 256 at 8x8, 3 x 512 at 4x4; the configuration text says
15, its enumeration gives 14) are chained inside each stage: F(4x4,3x3) Legendre
int8 with ReLU, the int8 output codes of one layer (scale s_y) being the input
codes of the next.  A stage starts from a fresh seeded tensor, because the
stride-2 layers that change the resolution are not part of the list.  The stem's
3 input channels are zero-padded to 16 (the library's channel granularity).
Every layer's V, U, M and int8 y must equal the oracle's bit for bit, so any
drift would show at the layer where it starts.  The chain runs at a reduced
batch (N = 32) and at the configuration's own N = 256, the size the benchmark
times; there each layer is also run the way the benchmark runs it (filters
transformed beforehand, fused = AUTO, which picks the kernels by layer shape).
"""
import numpy as np
import pytest

import synth_inputs as si
from helpers import assert_layer_parity, gpu_layer, oracle_layer

pytestmark = pytest.mark.gpu


def stage_layers():
    stages = {}
    for (C, K, HW) in si.RESNET18_STACK:
        stages.setdefault(HW, []).append((C, K))
    return stages


def run_as_benchmark(xq, wq, scales):
    """One layer through wino_conv2d with pretransformed filters and fused = AUTO, int8 + ReLU
    output: returns y."""
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = xq.shape
    K = wq.shape[0]
    sc = wn.Scales.from_dict(scales)
    x = torch.from_numpy(np.ascontiguousarray(xq, dtype=np.int8)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq, dtype=np.int8)).to(dev)
    layout = wn.wino_preferred_operand_layout(wn.ConvDesc(N, H, W, C, K, m=4, out_type=wn.OUT_I8,
                                                          relu=1))
    desc = wn.ConvDesc(N, H, W, C, K, m=4, out_type=wn.OUT_I8, relu=1, operand_layout=layout)
    V = torch.empty((wn.wino_operand_bytes(desc)[0],), dtype=torch.int8, device=dev)
    wn.wino_weight_transform(desc, w, V, sc)
    run = wn.ConvDesc(N, H, W, C, K, m=4, out_type=wn.OUT_I8, relu=1, weights_pretransformed=1,
                      fused=wn.FUSED_AUTO, operand_layout=layout)
    ws = torch.empty(wn.wino_workspace_bytes(run), dtype=torch.uint8, device=dev)
    y = torch.full((N, H, W, K), 77, dtype=torch.int8, device=dev)
    wn.wino_conv2d(run, x, V, y, sc, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("N", [32, 256])
@pytest.mark.parametrize("HW", [32, 16, 8, 4])
def test_chain_within_stage(HW, N):
    layers = stage_layers()[HW]
    rng_seed = 4
    C0 = layers[0][0]
    x, _ = si.make_real(N, HW, HW, C0, 1, seed=rng_seed)
    if C0 % 16:
        x = np.concatenate([x, np.zeros(x.shape[:3] + (16 - C0 % 16,), np.float32)], axis=3)
    xq, s_x = si.cast_int8(x)
    for li, (C, K) in enumerate(layers):
        _, w = si.make_real(1, 1, 1, C, K, seed=rng_seed * 100 + HW + li)
        if C % 16:
            w = np.concatenate([w, np.zeros((K, 16 - C % 16, 3, 3), np.float32)], axis=1)
        wq, s_w = si.cast_int8(w)
        kw = dict(m=4, base="legendre", out_type="i8", relu=True)
        ora, sc = oracle_layer(xq, wq, s_x, s_w, **kw)
        got = gpu_layer(xq, wq, sc, whole=True, **kw)
        assert_layer_parity(ora, got, "i8")
        assert got["y"].min() >= 0
        if N == 256:
            assert np.array_equal(run_as_benchmark(xq, wq, sc).astype(np.int64), ora["y"])
        xq, s_x = got["y"], sc["s_y"]           # the GPU's own output feeds the next layer
