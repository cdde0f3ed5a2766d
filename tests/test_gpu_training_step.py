"""The pieces a Winograd-aware training step of one flex layer needs, chained through the C
ABI: device-side calibration, forward pass, backward pass, and a host-side update of the
three matrices.  The same loop runs in the oracle (tests/test_oracle_backward.py); here the
library's losses must follow the oracle's and the error of the quantised layer must shrink."""
import numpy as np
import pytest

from helpers import small_layer
from oracle import backward as bw
from oracle import direct, flex, quantised as q

pytestmark = pytest.mark.gpu


def test_gradient_steps_on_the_flex_matrices_through_the_library():
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    m, base = 4, "legendre"
    N, H, W, C, K = 2, 8, 8, 16, 16
    n = m + 2
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=5)
    y_ref = direct.direct_conv(xq.astype(np.float64) * float(s_x), wq.astype(np.float64) * float(s_w))
    rng = np.random.default_rng(0)
    start = flex.FlexMatrices.from_exact(m, base=base)
    for name in ("GP", "BPT", "APT"):
        a = getattr(start, name)
        setattr(start, name, (a + 0.03 * rng.standard_normal(a.shape) * np.abs(a).max()).astype(np.float32))

    def update(fm, grads):
        for name in ("GP", "BPT", "APT"):
            a, d = getattr(fm, name).astype(np.float64), grads["d" + name].astype(np.float64)
            step = 0.05 * np.abs(a).max() / max(np.abs(d).max(), 1e-30)
            setattr(fm, name, (a - step * d).astype(np.float32))

    # oracle loop
    cfg = q.LayerConfig(m=m, base=base, bits_hadamard=9, inner_quant=True, out_type="f32")
    fm = flex.FlexMatrices(start.GP.copy(), start.BPT.copy(), start.APT.copy())
    ref_losses = []
    for _ in range(5):
        fwd, sc = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm)
        y = fwd["y"].astype(np.float64)
        ref_losses.append(0.5 * float(((y - y_ref) ** 2).mean()))
        f = lambda name: float(sc[name])
        update(fm, bw.flex_backward((y - y_ref) / y_ref.size, wq.astype(np.float64) * f("s_w"),
                                    fwd["X1"].astype(np.float64) * f("s_x1"),
                                    fwd["M1"].astype(np.float64) * f("s_m1"),
                                    bw.dequantise(fwd["U"], f("s_u")), bw.dequantise(fwd["V"], f("s_v")),
                                    fm, xq.shape, m, base))

    # library loop
    desc = wn.ConvDesc(N, H, W, C, K, m=m, base=wn.BASE_LEGENDRE, bits_hadamard=9)
    n2, T = desc.n ** 2, desc.tiles
    x = torch.from_numpy(xq).to(dev)
    w = torch.from_numpy(wq).to(dev)
    yref_d = torch.from_numpy(y_ref.astype(np.float32)).to(dev)
    y = torch.empty((N, H, W, K), dtype=torch.float32, device=dev)
    U = torch.empty((n2, T, C), dtype=torch.int8, device=dev)
    V = torch.empty((n2, K, C), dtype=torch.int8, device=dev)
    M = torch.empty((n2, T, K), dtype=torch.int16, device=dev)
    dx = torch.empty((N, H, W, C), dtype=torch.float32, device=dev)
    dw = torch.empty((K, C, 3, 3), dtype=torch.float32, device=dev)
    dGP = torch.empty((n, 3), dtype=torch.float32, device=dev)
    dBPT = torch.empty((n, n), dtype=torch.float32, device=dev)
    dAPT = torch.empty((m, n), dtype=torch.float32, device=dev)
    cws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    bws = torch.empty(wn.wino_flex_backward_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    fm = flex.FlexMatrices(start.GP.copy(), start.BPT.copy(), start.APT.copy())
    losses = []
    for _ in range(5):
        gfm = wn.FlexMatrices(fm.GP, fm.BPT, fm.APT)
        sc = wn.wino_flex_calibrate(desc, gfm, x, w, None, float(s_x), float(s_w), cws)
        wn.wino_flex_weight_transform(desc, gfm, w, V, sc)
        wn.wino_flex_input_transform(desc, gfm, x, U, sc)
        wn.wino_contract(desc, U, V, M, sc)
        wn.wino_flex_output_transform(desc, gfm, M, y, sc)
        diff = y - yref_d                                   # the loss and its gradient: caller's code
        losses.append(0.5 * float((diff.double() ** 2).mean()))
        dy = (diff / diff.numel()).contiguous()
        wn.wino_flex_backward(desc, gfm, dy, x, w, U, V, M, sc, dx, dw, dGP, dBPT, dAPT, bws)
        torch.cuda.synchronize()
        update(fm, {"dGP": dGP.cpu().numpy(), "dBPT": dBPT.cpu().numpy(), "dAPT": dAPT.cpu().numpy()})

    assert losses[0] == pytest.approx(ref_losses[0], rel=1e-6)      # same matrices: same forward pass
    # later steps: the fp32 gradients differ from the fp64 ones in their last bits, so the updated
    # fp32 matrices may differ by an ulp and a few codes may flip; the losses stay close
    assert np.allclose(losses, ref_losses, rtol=2e-2), (losses, ref_losses)
    assert min(losses[3:]) < 0.6 * losses[0], losses
