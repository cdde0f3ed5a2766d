"""wino_conv2d under HIP graph capture: it allocates nothing, never synchronises
and queues only kernels, so a captured layer must replay to the eager result.
The graph is replayed several times with eager work and synchronisations in
between, and every replay is compared with the eager output."""
import numpy as np
import pytest

from helpers import oracle_layer, small_layer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fused", [0, 1])
def test_captured_layer_replays_to_the_eager_result(fused):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    xq, wq, s_x, s_w = small_layer(4, 8, 8, 64, 64, seed=110)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, m=4, base="legendre", out_type="i8", relu=True)
    desc = wn.ConvDesc(4, 8, 8, 64, 64, m=4, out_type=wn.OUT_I8, relu=1, fused=fused)
    scales = wn.Scales.from_dict(sc)
    x = torch.from_numpy(xq).to(dev)
    w = torch.from_numpy(wq).to(dev)
    y = torch.zeros((4, 8, 8, 64), dtype=torch.int8, device=dev)
    ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        wn.wino_conv2d(desc, x, w, y, scales, ws, s)             # eager warm-up on the side stream
        torch.cuda.synchronize()
        eager = y.clone()
        assert np.array_equal(eager.cpu().numpy().astype(np.int64), ora["y"])
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            wn.wino_conv2d(desc, x, w, y, scales, ws, s)
    for rep in range(4):
        y.fill_(rep + 1)                                         # eager work between replays
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager), "replay %d differs" % rep
        # new input values through the same graph
    x2 = torch.roll(x, 1, dims=0)
    x.copy_(x2)
    g.replay()
    torch.cuda.synchronize()
    ora2, _ = oracle_layer(np.roll(xq, 1, axis=0), wq, s_x, s_w, m=4, base="legendre",
                           out_type="i8", relu=True)
    # the scales were calibrated on the same multiset of images, so they are unchanged
    assert np.array_equal(y.cpu().numpy().astype(np.int64), ora2["y"])


def test_peak_probes_run_and_report_their_work():
    import torch
    import paper_2004_11077_amd as wn
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    assert wn.wino_probe_peak(wn.PROBE_MFMA_I8, 8, 16, sink) == 8 * 4 * 16 * 4 * 2 * 32 ** 3
    assert wn.wino_probe_peak(wn.PROBE_VALU_MAD24, 8, 16, sink) == 8 * 256 * 16 * 8
    assert wn.wino_probe_peak(wn.PROBE_MFMA_BF16, 8, 16, sink) == 8 * 4 * 16 * 4 * 2 * 32 * 32 * 16
    torch.cuda.synchronize()
    assert int(sink.item()) == 0


def test_captured_backward_replays_to_the_eager_result():
    """wino_backward queues kernels only (no allocation, no memset, no synchronisation)."""
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K, m = 3, 9, 8, 48, 80, 4
    rng = np.random.default_rng(31)
    desc = wn.ConvDesc(N, H, W, C, K, m=m)
    n2, T = desc.n ** 2, desc.tiles
    dy = torch.from_numpy(rng.standard_normal((N, H, W, K)).astype(np.float32)).to(dev)
    U = torch.from_numpy(rng.integers(-127, 128, (n2, T, C)).astype(np.int8)).to(dev)
    V = torch.from_numpy(rng.integers(-127, 128, (n2, K, C)).astype(np.int8)).to(dev)
    sc = wn.Scales.from_dict({"s_u": 0.02, "s_v": 0.01})
    dx = torch.zeros((N, H, W, C), dtype=torch.float32, device=dev)
    dw = torch.zeros((K, C, 3, 3), dtype=torch.float32, device=dev)
    ws = torch.empty(wn.wino_backward_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        wn.wino_backward(desc, dy, U, V, sc, dx, dw, ws, s)
        torch.cuda.synchronize()
        eager_dx, eager_dw = dx.clone(), dw.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            wn.wino_backward(desc, dy, U, V, sc, dx, dw, ws, s)
    for rep in range(3):
        dx.fill_(float(rep + 1))
        dw.fill_(-1.0)
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(dx, eager_dx) and torch.equal(dw, eager_dw), "replay %d differs" % rep
