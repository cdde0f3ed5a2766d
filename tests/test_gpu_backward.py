"""Backward pass of one layer: library (fp32, through the C ABI) against the fp64 oracle.

Tolerance.  Every result is a chain of fp32 sums of products: two short
brackets (at most 8 terms each) around one contraction of length L (K for the
input gradient, T for the weight gradient).  With unit roundoff u = 2^-24 the
error of such a sum is at most about (L + 16) u sum|terms|, and for the
zero-mean synthetic gradients used here it behaves like sqrt(L) u times the
largest result.  The tests allow 1e-5 of the largest reference value for the
brackets and contractions with L <= 512, and 3e-5 at L = T = 1024 (the headline
shape), i.e. a few sqrt(L) u.
"""
import numpy as np
import pytest

from oracle import backward as bw

pytestmark = pytest.mark.gpu


def run_backward(dy, Uq, Vq, shape, m, scales):
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C, K = shape
    desc = wn.ConvDesc(N, H, W, C, K, m=m)
    n2, T = desc.n ** 2, desc.tiles
    nbytes = wn.wino_backward_workspace_bytes(desc)
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device=dev)
    dx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device=dev)
    dw = torch.full((K, C, 3, 3), float("nan"), dtype=torch.float32, device=dev)
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(dev)
    wn.wino_backward(desc, t(dy, np.float32), t(Uq, np.int8), t(Vq, np.int8),
                     wn.Scales.from_dict(scales), dx, dw, ws)
    torch.cuda.synchronize()
    r64 = lambda v: (v + 63) // 64 * 64            # 256-byte rounding, in floats
    out, o = {}, 0
    for name, shp in (("dM", (n2, T, K)), ("dU", (n2, T, C)), ("dV", (n2, K, C))):
        cnt = int(np.prod(shp))
        out[name] = ws[o:o + cnt].reshape(shp).cpu().numpy()
        o += r64(cnt)
    out["dx"], out["dw"] = dx.cpu().numpy(), dw.cpu().numpy()
    return out


def reference(dy, Uq, Vq, shape, m, scales):
    if hasattr(scales["s_u"], "__len__"):             # per-point scales
        U = bw.dequantise(Uq, None, scales["s_u"])
        V = bw.dequantise(Vq, None, scales["s_v"])
    else:
        U, V = bw.dequantise(Uq, scales["s_u"]), bw.dequantise(Vq, scales["s_v"])
    return bw.backward_layer(dy.astype(np.float64), U, V, shape[:4], m)


def make_case(shape, m, seed, per_point):
    N, H, W, C, K = shape
    rng = np.random.default_rng(seed)
    n2 = (m + 2) ** 2
    T = N * (-(-H // m)) * (-(-W // m))
    dy = rng.standard_normal((N, H, W, K)).astype(np.float32)
    Uq = rng.integers(-127, 128, (n2, T, C)).astype(np.int8)
    Vq = rng.integers(-127, 128, (n2, K, C)).astype(np.int8)
    if per_point:
        pt = lambda: [float(v) for v in rng.uniform(0.005, 0.05, n2).astype(np.float32)]
        scales = {"s_u": pt(), "s_v": pt()}
    else:
        scales = {"s_u": 0.02, "s_v": 0.011}
    return dy, Uq, Vq, scales


def check(ref, got, tol):
    for key in ("dM", "dU", "dV", "dx", "dw"):
        assert got[key].shape == ref[key].shape, key
        assert np.isfinite(got[key]).all(), key + " holds values the kernels did not write"
        if ref[key].size == 0:
            continue
        bound = tol * max(float(np.abs(ref[key]).max()), 1e-30)
        err = float(np.abs(got[key].astype(np.float64) - ref[key]).max())
        assert err <= bound, "%s: max abs err %g > %g" % (key, err, bound)


CASES = [
    # m, (N, H, W, C, K), per_point
    (4, (2, 8, 8, 16, 16), False),
    (4, (3, 11, 6, 48, 80), True),          # ragged image, ragged 64-blocks in every GEMM dimension
    (4, (1, 13, 5, 256, 64), False),
    (2, (2, 7, 9, 32, 16), True),
    (2, (5, 6, 6, 64, 144), False),
    (6, (1, 12, 12, 16, 32), False),
    (6, (2, 7, 8, 32, 16), True),
    (4, (40, 4, 4, 16, 32), False),         # T = 40: reduction over tiles not a multiple of 32
    (4, (64, 16, 16, 16, 16), False),       # T = 1024, few outputs: dV summed from 8 ranges of tiles
    (2, (64, 16, 16, 16, 16), False),       # T = 4096: 16 ranges, added by a kernel of their own
    (2, (37, 12, 12, 32, 16), True),        # T = 1332: 8 ranges, the last one ragged
    (4, (37, 12, 12, 16, 32), False),       # T = 333: 2 ranges of 6 and 5 chunks, the last chunk ragged
]


@pytest.mark.parametrize("m,shape,per_point", CASES)
def test_backward_matches_oracle(m, shape, per_point):
    dy, Uq, Vq, scales = make_case(shape, m, seed=900 + m + shape[3], per_point=per_point)
    got = run_backward(dy, Uq, Vq, shape, m, scales)
    # 1e-5 up to reductions of 512 terms, sqrt(L)-scaled beyond (docstring)
    T = shape[0] * (-(-shape[1] // m)) * (-(-shape[2] // m))
    check(reference(dy, Uq, Vq, shape, m, scales), got, 1e-5 * max(1.0, (T / 512.0) ** 0.5))


def test_dv_parts_of_the_shapes_above():
    import paper_2004_11077_amd as wn
    parts = lambda m, s: wn.wino_backward_dv_parts(wn.ConvDesc(*s, m=m))
    assert parts(4, (64, 16, 16, 16, 16)) == 8 and parts(2, (37, 12, 12, 32, 16)) == 8
    assert parts(4, (37, 12, 12, 16, 32)) == 2 and parts(4, (256, 8, 8, 256, 256)) == 2
    assert parts(2, (64, 16, 16, 16, 16)) == 16


@pytest.mark.parametrize("shape", [(0, 8, 8, 16, 16), (2, 8, 8, 16, 0), (2, 8, 8, 0, 16), (2, 0, 8, 16, 16)])
def test_backward_empty_problems(shape):
    dy, Uq, Vq, scales = make_case(shape, 4, seed=1, per_point=False)
    got = run_backward(dy, Uq, Vq, shape, 4, scales)
    ref = reference(dy, Uq, Vq, shape, 4, scales)
    for key in ("dx", "dw"):
        assert got[key].shape == ref[key].shape
        assert np.array_equal(got[key], ref[key].astype(np.float32))   # all zero, or empty


def test_backward_after_the_library_forward_pass_headline_shape():
    """U and V produced by the forward kernels of the headline workload."""
    import synth_inputs as si
    from helpers import gpu_layer
    wl = si.WORKLOADS["cfg4a_f4_c256"]
    L = si.make_layer(wl)
    scales = si.workload_scales(wl.name)
    fwd = gpu_layer(L["xq"], L["wq"], scales, m=4, base="legendre")
    rng = np.random.default_rng(77)
    shape = (wl.N, wl.H, wl.W, wl.C, wl.K)
    dy = rng.standard_normal((wl.N, wl.H, wl.W, wl.K)).astype(np.float32)
    got = run_backward(dy, fwd["U"], fwd["V"], shape, 4, scales)
    ref = reference(dy, fwd["U"], fwd["V"], shape, 4, scales)
    check(ref, got, 3e-5)


def random_cases():
    rng = np.random.default_rng(4242)
    out = []
    for i in range(16):
        out.append((int(rng.choice([2, 4, 6])),
                    (int(rng.integers(1, 6)), int(rng.integers(1, 14)), int(rng.integers(1, 14)),
                     int(rng.choice([16, 32, 48, 80, 144, 272])), int(rng.choice([16, 32, 48, 80, 144]))),
                    bool(rng.integers(0, 2)), 7000 + i))
    return out


@pytest.mark.parametrize("m,shape,per_point,seed", random_cases(),
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_backward_random_shapes(m, shape, per_point, seed):
    """Seeded random shapes: ragged images, 64-blocks and 32-chunks with tails in every dimension."""
    dy, Uq, Vq, scales = make_case(shape, m, seed=seed, per_point=per_point)
    got = run_backward(dy, Uq, Vq, shape, m, scales)
    check(reference(dy, Uq, Vq, shape, m, scales), got, 1e-5)


ONE_TERM_CASES = [(4, (3, 12, 12, 80, 48)), (4, (5, 9, 9, 144, 272)), (2, (40, 4, 4, 16, 144))]


@pytest.mark.parametrize("m,shape", ONE_TERM_CASES)
def test_contractions_keep_all_24_bits_of_dM(m, shape):
    """The contractions multiply dM by the codes in pieces on a narrower matrix pipe; a dropped
    or misplaced piece would cost at least 2^-16 of a product, which the max-relative bound
    above cannot see.  With codes that leave ONE non-zero term in every reduction, each output
    is s * dM * code for a single dM value with a full 24-bit significand, and must agree with
    the fp64 product of the library's own dM to a few units of fp32 roundoff, element by
    element."""
    N, H, W, C, K = shape
    rng = np.random.default_rng(31 + C)
    n2 = (m + 2) ** 2
    T = N * (-(-H // m)) * (-(-W // m))
    dy = rng.standard_normal((N, H, W, K)).astype(np.float32)
    Uq = np.zeros((n2, T, C), dtype=np.int8)
    Vq = np.zeros((n2, K, C), dtype=np.int8)
    code = lambda size: (rng.integers(1, 128, size) * rng.choice([-1, 1], size)).astype(np.int8)
    t0 = rng.integers(0, T, (n2, C))                 # the one tile with a non-zero code of U, per (p, c)
    k0 = rng.integers(0, K, (n2, C))                 # the one output channel with a non-zero code of V
    p_idx, c_idx = np.meshgrid(np.arange(n2), np.arange(C), indexing="ij")
    Uq[p_idx, t0, c_idx] = code((n2, C))
    Vq[p_idx, k0, c_idx] = code((n2, C))
    scales = {"s_u": 0.02, "s_v": 0.011}
    got = run_backward(dy, Uq, Vq, shape, m, scales)
    dM = got["dM"].astype(np.float64)                # [n2, T, K], exact fp32 values
    s_u, s_v = float(np.float32(scales["s_u"])), float(np.float32(scales["s_v"]))
    dU_ref = dM[p_idx[:, None, :], np.arange(T)[None, :, None], k0[:, None, :]] * \
        Vq[p_idx, k0, c_idx].astype(np.float64)[:, None, :] * s_v          # [n2, T, C]
    dV_ref = dM[p_idx[:, None, :], t0[:, None, :], np.arange(K)[None, :, None]] * \
        Uq[p_idx, t0, c_idx].astype(np.float64)[:, None, :] * s_u          # [n2, K, C]
    for name, ref in (("dU", dU_ref), ("dV", dV_ref)):
        err = np.abs(got[name].astype(np.float64) - ref)
        assert (err <= 4 * 2.0 ** -24 * np.abs(ref)).all(), \
            "%s: worst relative error %g" % (name, float((err / np.maximum(np.abs(ref), 1e-300)).max()))


def test_backward_scales_exactly_with_powers_of_two():
    """Scaling dy by a power of two must scale every result by exactly that power (no piece
    of the split operands under- or overflows within 2^-40 ... 2^40)."""
    m, shape = 4, (3, 11, 6, 144, 80)
    dy, Uq, Vq, scales = make_case(shape, m, seed=5, per_point=False)
    base = run_backward(dy, Uq, Vq, shape, m, scales)
    for e in (-40, 40):
        f = np.float32(2.0 ** e)
        got = run_backward(dy * f, Uq, Vq, shape, m, scales)
        for key in ("dM", "dU", "dV", "dx", "dw"):
            assert np.array_equal(got[key], base[key] * f), (key, e)
