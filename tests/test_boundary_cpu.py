"""CPU-only checks of the C-ABI boundary: exports, host matrix builder, error paths.

No kernel is launched here; calls that would reach the GPU are only made with
arguments that the host-side validation rejects first.
"""
import ctypes as C
import os
import re
from fractions import Fraction

import pytest

from oracle import matrices as mx

wn = pytest.importorskip("paper_2004_11077_amd")
from paper_2004_11077_amd import binding  # noqa: E402

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(wn.lib_path()),
                                reason="libwino.so not built (python -m paper_2004_11077_amd.build)")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "wino.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wino_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = C.CDLL(wn.lib_path())
    names = declared_symbols()
    assert len(names) >= 11
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(binding.EXPORTS)


ORACLE_NAMES = {"G": "G", "BT": "BT", "AT": "AT", "PT": "PT", "PINVT": "PinvT", "GP": "GP",
                "BPT": "BPT", "APT": "APT"}


@pytest.mark.parametrize("m", [2, 4, 6])
def test_make_matrices_equals_oracle(m):
    got = wn.wino_make_matrices(m, 3, mx.POINTS[m], wn.BASE_LEGENDRE)
    ora = mx.Matrices(m, 3)
    for name, oname in ORACLE_NAMES.items():
        assert getattr(got, name) == getattr(ora, oname), name
        N, rho = got.int_form(name)
        assert (N, rho) == mx.int_form(getattr(ora, oname)), name


def test_make_matrices_canonical_base_has_identity_P():
    got = wn.wino_make_matrices(4, 3, mx.POINTS[4], wn.BASE_CANONICAL)
    assert got.PT == mx.identity(6) and got.PINVT == mx.identity(6)
    assert got.GP == got.G and got.BPT == got.BT and got.APT == got.AT


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("base,name", [(2, "chebyshev"), (3, "hermite")])
def test_make_matrices_other_bases(m, base, name):
    got = wn.wino_make_matrices(m, 3, mx.POINTS[m], base)
    ora = mx.Matrices(m, 3, base=name)
    for gname, oname in ORACLE_NAMES.items():
        assert getattr(got, gname) == getattr(ora, oname), gname


@pytest.mark.parametrize("m,r,pts", [(3, 2, [0, 1, -1]), (2, 5, [0, 1, -1, 2, -2]),
                                     (4, 3, [0, 1, -1, Fraction(1, 2), -2]), (1, 1, []),
                                     (3, 3, [0, 1, -1, Fraction(3, 2)])])
def test_make_matrices_other_sizes_and_points(m, r, pts):
    got = wn.wino_make_matrices(m, r, pts, wn.BASE_LEGENDRE)
    AT, G, BT = mx.toom_cook(m, r, pts)
    assert (got.AT, got.G, got.BT) == (AT, G, BT)
    PT = mx.legendre_PT(m + r - 1)
    assert got.PT == PT and got.PINVT == mx.inverse(PT)


def test_make_matrices_error_codes():
    for args, code in [((4, 3, [0, 1, 1, 2, -2]), -1),          # duplicate point
                       ((4, 3, [0, 1, -1]), -1),                 # wrong point count
                       ((0, 3, [0]), -1),                        # m < 1
                       ((7, 3, list(range(8))), -2),             # n = 9 > 8
                       ((6, 3, [0, 10**6, -10**6, 10**7, -10**7, 10**8, -10**8]), -3)]:
        with pytest.raises(wn.WinoError) as e:
            wn.wino_make_matrices(*args)
        assert e.value.code == code, args
    lib = binding._load()
    pts = (binding._Rat * 3)(binding._Rat(0, 1), binding._Rat(1, 0), binding._Rat(2, 1))
    h = C.c_void_p()
    assert lib.wino_make_matrices(2, 3, pts, 3, 1, C.byref(h)) == -1      # zero denominator
    assert b"denominator" in lib.wino_last_error()
    assert lib.wino_make_matrices(2, 3, pts, 3, 1, None) == -1


def test_workspace_bytes_and_descriptor_validation():
    d = wn.ConvDesc(256, 8, 8, 256, 256, m=4)
    n2, T = 36, 1024
    r256 = lambda v: (v + 255) // 256 * 256
    assert wn.wino_workspace_bytes(d) == r256(n2 * 256 * 256) + 2 * r256(n2 * T * 256)
    d9 = wn.ConvDesc(256, 8, 8, 256, 256, m=4, bits_hadamard=9, weights_pretransformed=1)
    assert wn.wino_workspace_bytes(d9) == r256(n2 * T * 256) + r256(n2 * T * 256 * 2)
    for kw, code in [(dict(m=3), -2), (dict(m=4, r=5), -2), (dict(bits_hadamard=7), -2),
                     (dict(bits_in=16), -2), (dict(bits_in=32, out_type=wn.OUT_I8), -2), (dict(base=5), -1), (dict(out_type=9), -1),
                     (dict(out_type=wn.OUT_I32), -2),            # Legendre has no integer A_P^T
                     (dict(m=6, base=wn.BASE_CANONICAL, out_type=wn.OUT_I32), -2)]:
        with pytest.raises(wn.WinoError) as e:
            wn.wino_workspace_bytes(wn.ConvDesc(1, 8, 8, 16, 16, **kw))
        assert e.value.code == code, kw
    for shape in [(1, 8, 8, 12, 16), (1, 8, 8, 16, 24), (-1, 8, 8, 16, 16)]:
        with pytest.raises(wn.WinoError) as e:
            wn.wino_workspace_bytes(wn.ConvDesc(*shape))
        assert e.value.code == -1
    with pytest.raises(wn.WinoError) as e:                       # C too large for exact fp32
        wn.wino_workspace_bytes(wn.ConvDesc(1, 8, 8, 2048, 16, bits_hadamard=32))
    assert e.value.code == -3


def test_stage_calls_reject_bad_arguments_before_any_launch():
    lib = binding._load()
    d = wn.ConvDesc(1, 8, 8, 16, 16)
    s = wn.Scales.from_dict({})
    assert lib.wino_input_transform(C.byref(d), None, None, C.byref(s), None) == -1
    assert b"null pointer" in lib.wino_last_error()
    bad = wn.Scales.from_dict({"s_u": 0.0})
    fake = C.c_void_p(4096)      # never dereferenced: the scale check fails first
    assert lib.wino_input_transform(C.byref(d), fake, fake, C.byref(bad), None) == -1
    assert lib.wino_contract(C.byref(d), C.c_void_p(4100), fake, fake, C.byref(s), None) == -1
    assert b"aligned" in lib.wino_last_error()
    assert lib.wino_conv2d(C.byref(d), fake, fake, fake, C.byref(s), fake, 16, None) == -4
    dfused = wn.ConvDesc(1, 8, 8, 16, 16, bits_hadamard=32, fused=1)   # M on chip needs a cast M
    assert lib.wino_conv2d(C.byref(dfused), fake, fake, fake, C.byref(s), fake, 1 << 30, None) == -2
    assert lib.wino_contract_output(C.byref(dfused), fake, fake, fake, C.byref(s), None) == -2
    assert lib.wino_contract_output(C.byref(d), fake, fake, None, C.byref(s), None) == -1


def test_no_alloc_call_rejects_oversized_layers_before_touching_the_device():
    lib = binding._load()
    fake = C.c_void_p(4096)
    s = wn.Scales.from_dict({})
    big = wn.ConvDesc(1024, 32, 32, 64, 64, m=4)
    assert wn.wino_workspace_bytes(big) > wn.NOALLOC_MAX_BYTES
    assert lib.wino_conv2d_noalloc(C.byref(big), fake, fake, fake, C.byref(s), None) == -4
    assert b"scratch" in lib.wino_last_error()
    bad = wn.ConvDesc(1, 8, 8, 12, 16)
    assert lib.wino_conv2d_noalloc(C.byref(bad), fake, fake, fake, C.byref(s), None) == -1


def test_kernel_selection_and_workspace_of_the_whole_layer_call():
    """Which launches wino_conv2d makes, and the workspace that goes with them."""
    n2, T = 36, 1024
    r256 = lambda v: (v + 255) // 256 * 256
    V, U, M = r256(n2 * 256 * 256), r256(n2 * T * 256), r256(n2 * T * 256)
    wide = dict(m=4)
    cases = [
        (wn.FUSED_OFF, {}, ["operand_transforms", "contraction", "output_transform"], V + U + M),
        (wn.FUSED_AUTO, {}, ["operand_transforms", "contraction_output"], V + U),
        (wn.FUSED_AUTO, dict(bits_hadamard=9), ["operand_transforms", "contraction_output"], V + U),
        (wn.FUSED_ON, {}, ["operand_transforms", "contraction_output"], V + U),
        (wn.FUSED_AUTO, dict(weights_pretransformed=1, operand_layout=wn.LAYOUT_FRAGMENTS),
         ["input_transform", "contraction_output"], U),
        # a pretransformed V in rows is slow in the two-kernel form: AUTO runs one kernel per stage
        (wn.FUSED_AUTO, dict(weights_pretransformed=1), ["input_transform", "contraction",
                                                         "output_transform"], U + M),
        (wn.FUSED_ON, dict(weights_pretransformed=1), ["input_transform", "contraction_output"], U),
        (wn.FUSED_AUTO, dict(bits_hadamard=32), ["operand_transforms", "contraction",
                                                 "output_transform"], V + U + 4 * M),
    ]
    for mode, kw, names, ws in cases:
        d = wn.ConvDesc(256, 8, 8, 256, 256, fused=mode, **wide, **kw)
        assert wn.wino_conv2d_launches(d) == names, (mode, kw)
        assert wn.wino_workspace_bytes(d) == ws, (mode, kw)
    narrow = wn.ConvDesc(128, 32, 32, 64, 64, m=4, fused=wn.FUSED_AUTO)
    assert wn.wino_conv2d_launches(narrow) == ["weight_transform", "fused_layer"]
    assert wn.wino_workspace_bytes(narrow) == r256(36 * 64 * 64)
    few = wn.ConvDesc(256, 4, 4, 512, 512, m=4, fused=wn.FUSED_AUTO)   # 8 x 16 blocks: too few
    assert wn.wino_conv2d_launches(few) == ["operand_transforms", "contraction", "output_transform"]
    # up to 128 input channels AUTO keeps M on chip whenever the grid is not tiny, raw filters too
    for shape in [(256, 16, 16, 128, 128), (2048, 16, 16, 128, 128), (256, 16, 16, 64, 128)]:
        d = wn.ConvDesc(*shape, m=4, fused=wn.FUSED_AUTO)
        assert wn.wino_conv2d_launches(d) == ["operand_transforms", "contraction_output"], shape
    tiny = wn.ConvDesc(2, 8, 8, 128, 32, m=4, fused=wn.FUSED_AUTO)     # one block
    assert wn.wino_conv2d_launches(tiny) == ["operand_transforms", "contraction", "output_transform"]
    # 256 channels, 8-bit M: only where the grid is about one work group per compute unit
    pre = dict(m=4, fused=wn.FUSED_AUTO, weights_pretransformed=1, operand_layout=wn.LAYOUT_FRAGMENTS)
    assert wn.wino_conv2d_launches(wn.ConvDesc(256, 8, 8, 256, 256, **pre))[-1] == "contraction_output"
    for n_img, last in [(128, "output_transform"), (192, "contraction_output"), (320, "output_transform")]:
        raw = wn.ConvDesc(n_img, 8, 8, 256, 256, m=4, fused=wn.FUSED_AUTO)
        assert wn.wino_conv2d_launches(raw)[-1] == last, n_img
    big = wn.ConvDesc(512, 8, 8, 256, 256, m=4, fused=wn.FUSED_AUTO)
    assert wn.wino_preferred_operand_layout(big) == wn.LAYOUT_ROWS      # a larger grid: stage by stage
    # ... but a V that is handed over in fragment order is read by the form that can read it
    assert wn.wino_conv2d_launches(wn.ConvDesc(512, 8, 8, 256, 256, **pre))[-1] == "contraction_output"
    # ... with a 9-bit M at any size, but not beyond 256 channels
    h9 = dict(m=4, fused=wn.FUSED_AUTO, bits_hadamard=9)
    assert wn.wino_conv2d_launches(wn.ConvDesc(4096, 8, 8, 256, 256, **h9))[-1] == "contraction_output"
    assert wn.wino_conv2d_launches(wn.ConvDesc(256, 8, 8, 512, 512, **h9))[-1] == "output_transform"
    f6 = wn.ConvDesc(2, 8, 8, 32, 32, m=6, fused=wn.FUSED_ON)          # no single kernel for F(6,3)
    assert wn.wino_conv2d_launches(f6) == ["operand_transforms", "contraction_output"]
    assert wn.wino_conv2d_launches(wn.ConvDesc(0, 8, 8, 16, 16)) == []
    # fragment order pads tiles to 16 and channels to 64
    fr = wn.ConvDesc(3, 9, 7, 48, 80, m=4, operand_layout=wn.LAYOUT_FRAGMENTS)       # T = 18
    assert wn.wino_operand_bytes(fr) == (36 * 5 * 1 * 1024, 36 * 2 * 1 * 1024)
    assert wn.wino_operand_bytes(wn.ConvDesc(3, 9, 7, 48, 80, m=4)) == (36 * 80 * 48, 36 * 18 * 48)
    assert wn.wino_preferred_operand_layout(wn.ConvDesc(256, 8, 8, 256, 256)) == wn.LAYOUT_FRAGMENTS
    assert wn.wino_preferred_operand_layout(narrow) == wn.LAYOUT_ROWS
    with pytest.raises(wn.WinoError) as e:       # a V in fragment order needs the two-kernel form
        wn.wino_workspace_bytes(wn.ConvDesc(128, 32, 32, 64, 64, weights_pretransformed=1,
                                            operand_layout=wn.LAYOUT_FRAGMENTS))
    assert e.value.code == -2
    with pytest.raises(wn.WinoError) as e:
        wn.wino_workspace_bytes(wn.ConvDesc(1, 8, 8, 16, 16, operand_layout=5))
    assert e.value.code == -1
    wn.wino_set_option(wn.OPT_AUTO_CONOUT, 0)
    try:
        d = wn.ConvDesc(256, 8, 8, 256, 256, m=4, bits_hadamard=9, fused=wn.FUSED_AUTO)
        assert wn.wino_conv2d_launches(d) == ["operand_transforms", "contraction", "output_transform"]
    finally:
        wn.wino_set_option(wn.OPT_AUTO_CONOUT, 1)
    for opt, val in [(7, 0), (0, 1)]:
        with pytest.raises(wn.WinoError) as e:
            wn.wino_set_option(opt, val)
        assert e.value.code == -1


def test_flex_calls_validate_matrices_and_options_before_any_launch():
    import numpy as np
    lib = binding._load()
    s = wn.Scales.from_dict({})
    fake = C.c_void_p(4096)      # never dereferenced: validation fails first
    good = wn.FlexMatrices(np.ones((6, 3)), np.ones((6, 6)), np.ones((4, 6)))
    d = wn.ConvDesc(1, 8, 8, 16, 16)
    for mats, text in [(wn.FlexMatrices(np.full((6, 3), np.nan), np.ones((6, 6)), np.ones((4, 6))), b"GP"),
                       (wn.FlexMatrices(np.ones((6, 3)), np.full((6, 6), 3e6), np.ones((4, 6))), b"BPT"),
                       (wn.FlexMatrices(np.ones((6, 3)), np.ones((6, 6)), np.full((4, 6), np.inf)), b"APT")]:
        assert lib.wino_flex_input_transform(C.byref(d), C.byref(mats), fake, fake, C.byref(s), None) == -1
        assert text in lib.wino_last_error()
    assert lib.wino_flex_conv2d(C.byref(d), None, fake, fake, fake, C.byref(s), fake, 1 << 30, None) == -1
    for kw in (dict(inner_quant=0), dict(base=wn.BASE_CANONICAL, out_type=wn.OUT_I32), dict(bits_in=32),
               dict(fused=1)):
        dd = wn.ConvDesc(1, 8, 8, 16, 16, **kw)
        assert lib.wino_flex_conv2d(C.byref(dd), C.byref(good), fake, fake, fake, C.byref(s), fake,
                                    1 << 30, None) == -2, kw
    assert lib.wino_flex_conv2d(C.byref(d), C.byref(good), fake, fake, fake, C.byref(s), fake, 16, None) == -4
    assert lib.wino_flex_weight_transform(C.byref(d), C.byref(good), None, fake, C.byref(s), None) == -1
    assert lib.wino_flex_output_transform(C.byref(d), C.byref(good), fake, fake,
                                          C.byref(wn.Scales.from_dict({"s_m1": -1.0})), None) == -1


def test_probe_rejects_bad_arguments_before_any_launch():
    lib = binding._load()
    fake = C.c_void_p(4096)
    assert lib.wino_probe_peak(7, 1, 1, fake, None, None) == -1
    assert lib.wino_probe_peak(0, 0, 1, fake, None, None) == -1
    assert lib.wino_probe_peak(1, 1, 1 << 30, fake, None, None) == -1
    assert lib.wino_probe_peak(0, 1, 1, None, None, None) == -1


def test_per_point_scales_are_validated_before_any_launch():
    import numpy as np
    lib = binding._load()
    fake = C.c_void_p(4096)
    pp = wn.Scales.from_dict({"s_u": np.ones((6, 6)), "s_v": np.ones((6, 6)), "m_shift": [0] * 36})
    assert pp.per_point == 1
    for kw in (dict(bits_hadamard=32), dict(base=wn.BASE_CANONICAL, out_type=wn.OUT_I32)):
        d = wn.ConvDesc(1, 8, 8, 16, 16, **kw)
        assert lib.wino_contract(C.byref(d), fake, fake, fake, C.byref(pp), None) == -2, kw
    d = wn.ConvDesc(1, 8, 8, 16, 16)
    bad = wn.Scales.from_dict({"s_u": np.ones((6, 6)), "s_v": np.ones((6, 6)), "m_shift": [9] + [0] * 35})
    assert lib.wino_contract(C.byref(d), fake, fake, fake, C.byref(bad), None) == -1
    assert b"m_shift" in lib.wino_last_error()
    neg = wn.Scales.from_dict({"s_u": -np.ones((6, 6)), "s_v": np.ones((6, 6))})
    assert lib.wino_input_transform(C.byref(d), fake, fake, C.byref(neg), None) == -1
    fm = wn.FlexMatrices(np.ones((6, 3)), np.ones((6, 6)), np.ones((4, 6)))
    assert lib.wino_flex_input_transform(C.byref(d), C.byref(fm), fake, fake, C.byref(pp), None) == -2


def test_backward_workspace_and_argument_checks_before_any_launch():
    lib = binding._load()
    fake = C.c_void_p(4096)
    r256 = lambda v: (v + 255) // 256 * 256
    d = wn.ConvDesc(2, 8, 8, 32, 48)                     # F(4,3): n*n = 36, T = 8
    want = r256(36 * 8 * 48 * 4) + r256(36 * 8 * 32 * 4) + r256(36 * 48 * 32 * 4)
    assert wn.wino_backward_workspace_bytes(d) == want
    s = wn.Scales.from_dict({"s_u": 0.1, "s_v": 0.2})
    args = lambda desc, sc, ws=fake, nbytes=1 << 30: (
        C.byref(desc), fake, fake, fake, sc, fake, fake, ws, nbytes, None)
    assert lib.wino_backward(*args(wn.ConvDesc(2, 8, 8, 32, 48, bits_in=32), C.byref(s))) == -2
    assert lib.wino_backward(*args(d, None)) == -1                              # no scales
    assert lib.wino_backward(*args(d, C.byref(wn.Scales.from_dict({"s_u": 0.0, "s_v": 0.2})))) == -1
    assert lib.wino_backward(*args(d, C.byref(s), nbytes=want - 1)) == -4       # workspace too small
    assert lib.wino_backward(*args(d, C.byref(s), ws=C.c_void_p(4096 + 64))) == -4   # misaligned
    assert lib.wino_backward(*args(d, C.byref(s), ws=None)) == -1
    assert lib.wino_backward(C.byref(d), fake, C.c_void_p(4096 + 4), fake, C.byref(s), fake, fake, fake,
                             1 << 30, None) == -1                               # U not 16-byte aligned
    assert lib.wino_backward(C.byref(d), fake, fake, fake, C.byref(s), None, fake, fake, 1 << 30, None) == -1


def test_flex_backward_argument_checks_before_any_launch():
    import numpy as np
    lib = binding._load()
    fake = C.c_void_p(4096)
    r256 = lambda v: (v + 255) // 256 * 256
    d = wn.ConvDesc(2, 8, 8, 32, 48)                     # n*n = 36, T = 8
    tensors = r256(36 * 8 * 48 * 4) + 2 * r256(36 * 8 * 32 * 4) + r256(36 * 48 * 32 * 4)
    blocks = -(-8 * 48 // 256) + -(-8 * 32 // 256) + -(-48 * 32 // 256)
    assert wn.wino_flex_backward_workspace_bytes(d) == tensors + blocks * 256
    good = wn.FlexMatrices(np.ones((6, 3)), np.ones((6, 6)), np.ones((4, 6)))
    s = wn.Scales.from_dict({})
    grads = binding.FlexGrads(4096, 4096, 4096)

    def call(desc=d, fm=good, sc=s, gr=grads, ws=fake, nbytes=1 << 30, x=fake):
        return lib.wino_flex_backward(C.byref(desc), C.byref(fm) if fm is not None else None, fake, x,
                                      fake, fake, fake, fake, C.byref(sc) if sc is not None else None,
                                      fake, fake, C.byref(gr) if gr is not None else None, ws, nbytes, None)
    assert call(desc=wn.ConvDesc(2, 8, 8, 32, 48, bits_in=32)) == -2
    assert call(desc=wn.ConvDesc(2, 8, 8, 32, 48, inner_quant=0)) == -2       # Legendre flex needs the inner casts
    assert call(desc=wn.ConvDesc(0, 8, 8, 32, 48)) == -1                       # empty problem
    assert call(fm=None) == -1
    assert call(sc=None) == -1
    assert call(gr=None) == -1
    assert call(gr=binding.FlexGrads(4096, 0, 4096)) == -1
    assert call(x=None) == -1
    assert call(sc=wn.Scales.from_dict({"s_x1": 0.0})) == -1
    assert call(sc=wn.Scales.from_dict({"s_u": np.ones((6, 6)), "s_v": np.ones((6, 6))})) == -2   # per-point
    assert call(nbytes=tensors) == -4
    assert call(ws=C.c_void_p(4096 + 128)) == -4


def test_backward_dv_parts_and_their_workspace():
    r256 = lambda v: (v + 255) // 256 * 256
    # (shape, m) -> parts: fewer than 256 tiles of dV (128 outputs wide where K resp. C exceeds 64, else 64),
    # ranges of at least four 32-tile chunks
    cases = [((256, 8, 8, 256, 256), 4, 2), ((128, 32, 32, 64, 64), 4, 8), ((128, 16, 16, 128, 128), 4, 8),
             ((1, 8, 8, 16, 16), 4, 1), ((64, 16, 16, 16, 16), 4, 8), ((37, 12, 12, 16, 32), 4, 2),
             ((512, 16, 16, 16, 16), 2, 16)]
    for shape, m, parts in cases:
        d = wn.ConvDesc(*shape, m=m)
        assert wn.wino_backward_dv_parts(d) == parts, shape
        n2, T, (Cc, Kk) = d.n ** 2, d.tiles, shape[3:]
        assert wn.wino_backward_workspace_bytes(d) == (r256(n2 * T * Kk * 4) + r256(n2 * T * Cc * 4) +
                                                       r256(parts * n2 * Kk * Cc * 4))
    lib = binding._load()
    assert lib.wino_backward_dv_parts(C.byref(wn.ConvDesc(1, 8, 8, 16, 16)), None) == -1
    assert lib.wino_backward_dv_parts(C.byref(wn.ConvDesc(1, 8, 8, 17, 16)), C.byref(C.c_int())) == -1
