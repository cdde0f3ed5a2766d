"""GPU test of wino_conv2d_noalloc, the whole-layer call that takes no workspace and
allocates nothing (its scratch is a device array inside the library).

Its output must equal wino_conv2d's on the same inputs: bit for bit for int8 outputs, and for
fp32 outputs as well, since the same kernels run.  Two calls in a row share the built-in
scratch, the second on a smaller layer, so stale contents of the first must not leak into
the second; then a third, larger again, through another kernel selection.
"""
import numpy as np
import pytest

from helpers import oracle_layer, small_layer

pytestmark = pytest.mark.gpu


def both_ways(shape, seed, **kw):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=seed)
    ora, sc = oracle_layer(xq, wq, s_x, s_w, m=kw.get("m", 4), base="legendre",
                           bits_hadamard=kw.get("bits_hadamard", 8),
                           out_type="i8" if kw.get("out_type") == wn.OUT_I8 else "f32",
                           relu=bool(kw.get("relu", 0)))
    s = wn.Scales.from_dict(sc)
    x = torch.from_numpy(xq).to(dev)
    w = torch.from_numpy(wq).to(dev)
    desc = wn.ConvDesc(N, H, W, C, K, **kw)
    ydt = torch.int8 if kw.get("out_type") == wn.OUT_I8 else torch.float32
    y_ws = torch.full((N, H, W, K), 77, dtype=ydt, device=dev)
    y_na = torch.full((N, H, W, K), 55, dtype=ydt, device=dev)
    ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    wn.wino_conv2d(desc, x, w, y_ws, s, ws)
    wn.wino_conv2d_noalloc(desc, x, w, y_na, s)
    torch.cuda.synchronize()
    return ora["y"], y_ws.cpu().numpy(), y_na.cpu().numpy()


def test_no_alloc_call_equals_the_workspace_call_on_two_calls_in_a_row():
    import paper_2004_11077_amd as wn
    calls = [
        ((16, 16, 16, 128, 128), dict(m=4, out_type=wn.OUT_I8, relu=1, fused=wn.FUSED_OFF)),
        ((3, 9, 7, 48, 80), dict(m=4, out_type=wn.OUT_I8, relu=1, fused=wn.FUSED_OFF)),   # smaller
        ((8, 8, 8, 256, 256), dict(m=4, bits_hadamard=9, out_type=wn.OUT_F32, fused=wn.FUSED_ON)),
        ((2, 8, 8, 32, 32), dict(m=2, out_type=wn.OUT_F32, fused=wn.FUSED_ON)),           # smaller
    ]
    for i, (shape, kw) in enumerate(calls):
        ref, y_ws, y_na = both_ways(shape, 900 + i, **kw)
        assert np.array_equal(y_ws, y_na), (i, shape)
        if kw["out_type"] == wn.OUT_I8:
            assert np.array_equal(y_na.astype(np.int64), ref), (i, shape)
        else:
            assert np.abs(y_na - ref).max() <= 1e-5 * np.abs(ref).max(), (i, shape)


def test_no_alloc_call_rejects_layers_beyond_its_scratch():
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    desc = wn.ConvDesc(1024, 32, 32, 64, 64, m=4, fused=wn.FUSED_OFF)     # 65536 tiles: 300 MB
    assert wn.wino_workspace_bytes(desc) > wn.NOALLOC_MAX_BYTES
    t = torch.zeros(16, dtype=torch.int8, device=dev)
    with pytest.raises(wn.WinoError) as e:
        wn.wino_conv2d_noalloc(desc, t, t, t, wn.Scales.from_dict({}))
    assert e.value.code == -4 and "scratch" in str(e.value)
