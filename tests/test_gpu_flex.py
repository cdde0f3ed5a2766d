"""Parity of the flex layer (run-time fp32 matrices, Section 4.2) with oracle/flex.py.

Both sides evaluate the fp32 brackets in the same order with separately rounded
products and sums, so every integer tensor (V, U, M, int8 y) must agree bit for bit
and the fp32 output must agree exactly as well (asserted; the documented bar is
1e-5 of the output range)."""
import numpy as np
import pytest

from helpers import small_layer
from oracle import flex, quantised as q

pytestmark = pytest.mark.gpu


def noisy_matrices(m, base, seed, noise=0.05):
    rng = np.random.default_rng(seed)
    fm = flex.FlexMatrices.from_exact(m, base=base)
    for name in ("GP", "BPT", "APT"):
        a = getattr(fm, name)
        pert = noise * rng.standard_normal(a.shape) * np.abs(a).max()
        setattr(fm, name, (a + pert).astype(np.float32))
    return fm


def run_gpu(xq, wq, fm, scales, m, base, bits_hadamard, out_type, relu, whole):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = xq.shape
    K = wq.shape[0]
    desc = wn.ConvDesc(N, H, W, C, K, m=m,
                       base=wn.BASE_LEGENDRE if base == "legendre" else wn.BASE_CANONICAL,
                       bits_hadamard=bits_hadamard,
                       out_type=wn.OUT_I8 if out_type == "i8" else wn.OUT_F32, relu=int(relu))
    gfm = wn.FlexMatrices(fm.GP, fm.BPT, fm.APT)
    n2, T = desc.n ** 2, desc.tiles
    x = torch.from_numpy(np.ascontiguousarray(xq, dtype=np.int8)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq, dtype=np.int8)).to(dev)
    mdt = {8: torch.int8, 9: torch.int16, 32: torch.int32}[bits_hadamard]
    y = torch.full((N, H, W, K), 77, dtype=torch.int8 if out_type == "i8" else torch.float32,
                   device=dev)
    sc = wn.Scales.from_dict(scales)
    if whole:
        ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        wn.wino_flex_conv2d(desc, gfm, x, w, y, sc, ws)
        torch.cuda.synchronize()
        r256 = lambda v: (v + 255) // 256 * 256
        o = 0
        V = ws[o:o + n2 * K * C].view(torch.int8).reshape(n2, K, C); o += r256(n2 * K * C)
        U = ws[o:o + n2 * T * C].view(torch.int8).reshape(n2, T, C); o += r256(n2 * T * C)
        mb = n2 * T * K * torch.empty((), dtype=mdt).element_size()
        M = ws[o:o + mb].view(mdt).reshape(n2, T, K)
    else:
        V = torch.full((n2, K, C), 77, dtype=torch.int8, device=dev)
        U = torch.full((n2, T, C), 77, dtype=torch.int8, device=dev)
        M = torch.full((n2, T, K), 77, dtype=mdt, device=dev)
        wn.wino_flex_weight_transform(desc, gfm, w, V, sc)
        wn.wino_flex_input_transform(desc, gfm, x, U, sc)
        wn.wino_contract(desc, U, V, M, sc)
        wn.wino_flex_output_transform(desc, gfm, M, y, sc)
        torch.cuda.synchronize()
    return {"V": V.cpu().numpy(), "U": U.cpu().numpy(), "M": M.cpu().numpy(), "y": y.cpu().numpy()}


def check(ora, got, out_type):
    for key in ("V", "U", "M"):
        bad = np.nonzero(got[key].astype(np.int64) != ora[key])
        assert bad[0].size == 0, "%s: %d mismatches, first at %s" % (
            key, bad[0].size, [int(b[0]) for b in bad])
    if out_type == "i8":
        assert np.array_equal(got["y"].astype(np.int64), ora["y"]), "y codes differ"
    else:
        ref = ora["y"]
        tol = 1e-5 * max(float(np.abs(ref).max()), 1e-30)
        assert float(np.abs(got["y"].astype(np.float64) - ref).max()) <= tol
        assert np.array_equal(got["y"], ref.astype(np.float32)), "fp32 y not bit-identical"


CASES = [
    # m, base, shape (N,H,W,C,K), bits_hadamard, out_type, relu, whole
    (2, "canonical", (2, 8, 8, 16, 16), 8, "f32", False, False),
    (2, "legendre", (1, 7, 9, 16, 32), 9, "i8", True, True),
    (4, "canonical", (2, 8, 8, 32, 16), 32, "f32", True, False),
    (4, "legendre", (2, 8, 8, 32, 48), 8, "f32", False, False),
    (4, "legendre", (3, 10, 6, 48, 32), 9, "i8", True, True),
    (4, "legendre", (1, 13, 5, 16, 16), 32, "i8", False, False),
    (6, "canonical", (1, 12, 12, 16, 16), 8, "i8", False, True),
    (6, "legendre", (2, 8, 8, 16, 32), 8, "f32", True, False),
    (6, "legendre", (1, 7, 11, 32, 16), 9, "i8", True, True),
]


@pytest.mark.parametrize("m,base,shape,bh,out_type,relu,whole", CASES)
def test_flex_layer_matches_the_oracle(m, base, shape, bh, out_type, relu, whole):
    N, H, W, C, K = shape
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=200 + m + C)
    fm = noisy_matrices(m, base, seed=m * 7 + bh)
    cfg = q.LayerConfig(m=m, base=base, bits_hadamard=bh, out_type=out_type, relu=relu)
    ora, sc = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm)
    got = run_gpu(xq, wq, fm, sc, m, base, bh, out_type, relu, whole)
    check(ora, got, out_type)
    assert np.abs(ora["U"]).max() == 127 and np.abs(ora["V"]).max() == 127   # scales are tight


def test_exact_matrices_rounded_to_fp32_stay_close_to_the_static_layer():
    """Sanity link between the two variants on the GPU: the static rational matrices,
    rounded to fp32 and run through the flex kernels, give U within one step of the
    static kernels' U."""
    import torch
    import paper_2004_11077_amd as wn
    xq, wq, s_x, s_w = small_layer(2, 8, 8, 32, 32, seed=77)
    cfg = q.LayerConfig(m=4, base="legendre")
    ora, sc = q.run_layer(xq, wq, s_x, s_w, cfg)
    fm = flex.FlexMatrices.from_exact(4, base="legendre")
    got = run_gpu(xq, wq, fm, sc, 4, "legendre", 8, "f32", False, False)
    d = np.abs(got["U"].astype(np.int64) - ora["U"])
    assert d.max() <= 1 and np.mean(d != 0) < 0.02


@pytest.mark.parametrize("m,base,bh,out_type,relu", [(4, "legendre", 8, "i8", True),
                                                     (4, "canonical", 9, "f32", False),
                                                     (2, "legendre", 32, "i8", False),
                                                     (6, "legendre", 8, "f32", False)])
def test_flex_calibration_equals_the_oracles(m, base, bh, out_type, relu):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K = 2, 9, 8, 32, 16
    xq, wq, s_x, s_w = small_layer(N, H, W, C, K, seed=300 + m)
    fm = noisy_matrices(m, base, seed=m + 40)
    cfg = q.LayerConfig(m=m, base=base, bits_hadamard=bh, out_type=out_type, relu=relu)
    ora, sc = flex.run_layer_flex(xq, wq, s_x, s_w, cfg, fm)
    desc = wn.ConvDesc(N, H, W, C, K, m=m,
                       base=wn.BASE_LEGENDRE if base == "legendre" else wn.BASE_CANONICAL,
                       bits_hadamard=bh, out_type=wn.OUT_I8 if out_type == "i8" else wn.OUT_F32,
                       relu=int(relu))
    gfm = wn.FlexMatrices(fm.GP, fm.BPT, fm.APT)
    x = torch.from_numpy(np.ascontiguousarray(xq, dtype=np.int8)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq, dtype=np.int8)).to(dev)
    y = torch.zeros((N, H, W, K), dtype=torch.int8 if out_type == "i8" else torch.float32,
                    device=dev)
    cws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    got = wn.wino_flex_calibrate(desc, gfm, x, w, y, float(s_x), float(s_w), cws)
    torch.cuda.synchronize()
    for name, val in sc.items():
        assert np.float32(getattr(got, name)) == np.float32(val), name
    if out_type == "i8":
        assert np.array_equal(y.cpu().numpy().astype(np.int64), ora["y"])
    else:
        assert np.array_equal(y.cpu().numpy(), ora["y"].astype(np.float32))
