"""ctypes marshalling for libwino.so -- argument packing only, no arithmetic."""
import ctypes as C
import os
from fractions import Fraction

HERE = os.path.dirname(os.path.abspath(__file__))

BASE_CANONICAL, BASE_LEGENDRE, BASE_CHEBYSHEV, BASE_HERMITE = 0, 1, 2, 3
OUT_F32, OUT_I32, OUT_I8 = 0, 1, 2
FUSED_OFF, FUSED_ON, FUSED_AUTO = 0, 1, 2
LAYOUT_ROWS, LAYOUT_FRAGMENTS = 0, 1
MAT_NAMES = ("G", "BT", "AT", "PT", "PINVT", "GP", "BPT", "APT")
EXPORTS = ("wino_make_matrices", "wino_free_matrices", "wino_get_matrix", "wino_get_int_form",
           "wino_workspace_bytes", "wino_operand_bytes", "wino_preferred_operand_layout",
           "wino_calibrate_workspace_bytes", "wino_calibrate",
           "wino_conv2d", "wino_conv2d_noalloc", "wino_weight_transform",
           "wino_input_transform", "wino_transform_operands", "wino_contract",
           "wino_output_transform", "wino_contract_output", "wino_conv2d_launches",
           "wino_set_option", "wino_flex_weight_transform", "wino_flex_input_transform",
           "wino_flex_output_transform", "wino_flex_conv2d", "wino_flex_calibrate",
           "wino_backward_workspace_bytes", "wino_backward_dv_parts", "wino_backward",
           "wino_flex_backward_workspace_bytes", "wino_flex_backward",
           "wino_profile_next_launch", "wino_probe_peak", "wino_last_error")


class WinoError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libwino error %d: %s" % (code, text))
        self.code = code


class _Rat(C.Structure):
    _fields_ = [("num", C.c_int64), ("den", C.c_int64)]


class ConvDesc(C.Structure):
    """Mirror of wino_conv_desc_t."""
    _fields_ = [(n, C.c_int) for n in (
        "N", "H", "W", "C", "K", "m", "r", "base", "bits_in", "bits_hadamard", "inner_quant",
        "out_type", "relu", "weights_pretransformed", "fused", "operand_layout")]

    def __init__(self, N, H, W, C_, K, m=4, r=3, base=BASE_LEGENDRE, bits_in=8, bits_hadamard=8,
                 inner_quant=1, out_type=OUT_F32, relu=0, weights_pretransformed=0, fused=0,
                 operand_layout=0):
        super().__init__(N, H, W, C_, K, m, r, base, bits_in, bits_hadamard, inner_quant,
                         out_type, relu, weights_pretransformed, fused, operand_layout)

    @property
    def n(self):
        return self.m + self.r - 1

    @property
    def tiles(self):
        return self.N * (-(-self.H // self.m)) * (-(-self.W // self.m))


class Scales(C.Structure):
    """Mirror of wino_scales_t."""
    SCALARS = ("s_x", "s_x1", "s_u", "s_w", "s_w1", "s_v", "s_m", "s_m1", "s_y")
    _fields_ = ([(n, C.c_float) for n in SCALARS] +
                [("per_point", C.c_int), ("s_u_pt", C.c_float * 64), ("s_v_pt", C.c_float * 64),
                 ("m_shift", C.c_int * 64)])

    @classmethod
    def from_dict(cls, d):
        """Scalars by name; a sequence for "s_u" / "s_v" (with "m_shift") selects the
        per-point mode, as does "per_point": True on its own (for calibration)."""
        s = cls()
        s.per_point = int(bool(d.get("per_point", False)))
        for name in cls.SCALARS:
            v = d.get(name, 1.0)
            if name in ("s_u", "s_v") and hasattr(v, "__len__"):
                s.per_point = 1
                flat = [float(e) for row in v for e in (row if hasattr(row, "__len__") else [row])]
                arr = getattr(s, name + "_pt")
                for i in range(64):
                    arr[i] = flat[i] if i < len(flat) else 1.0
                v = 1.0
            setattr(s, name, float(v))
        if not hasattr(d.get("s_u", 1.0), "__len__"):
            for i in range(64):
                s.s_u_pt[i] = s.s_v_pt[i] = 1.0
        for i, v in enumerate(list(d.get("m_shift", []))[:64]):
            s.m_shift[i] = int(v)
        return s

    def to_dict(self, n):
        """Back to the oracle's naming; n = m + r - 1 gives the shape of per-point arrays."""
        out = {name: getattr(self, name) for name in self.SCALARS}
        if self.per_point:
            out["s_u"] = [[self.s_u_pt[i * n + j] for j in range(n)] for i in range(n)]
            out["s_v"] = [[self.s_v_pt[i * n + j] for j in range(n)] for i in range(n)]
            out["m_shift"] = [self.m_shift[i] for i in range(n * n)]
        return out


class FlexMatrices(C.Structure):
    """Mirror of wino_flex_matrices_t: host fp32 arrays GP [n,3], BPT [n,n], APT [m,n]."""
    _fields_ = [(n, C.POINTER(C.c_float)) for n in ("GP", "BPT", "APT")]

    def __init__(self, GP, BPT, APT):
        import numpy as np
        self._keep = [np.ascontiguousarray(a, dtype=np.float32) for a in (GP, BPT, APT)]
        super().__init__(*[a.ctypes.data_as(C.POINTER(C.c_float)) for a in self._keep])


class FlexGrads(C.Structure):
    """Mirror of wino_flex_grads_t: device fp32 arrays dGP [n,3], dBPT [n,n], dAPT [m,n]."""
    _fields_ = [(n, C.c_void_p) for n in ("dGP", "dBPT", "dAPT")]


def lib_path():
    return os.path.join(HERE, "libwino.so")


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("libwino.so is not built (run: python -m paper_2004_11077_amd.build); "
                          "there is no fallback path")
    # The tensors callers pass live in PyTorch's HIP runtime, and the first libamdhip64 loaded
    # under its SONAME serves the whole process: load PyTorch's first, so that the library's
    # kernels and the caller's memory and streams belong to one runtime whatever the import order.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    vp, ip = C.c_void_p, C.POINTER(C.c_int)
    lib.wino_last_error.restype = C.c_char_p
    lib.wino_make_matrices.argtypes = [C.c_int, C.c_int, C.POINTER(_Rat), C.c_int, C.c_int,
                                       C.POINTER(vp)]
    lib.wino_free_matrices.argtypes = [vp]
    lib.wino_free_matrices.restype = None
    lib.wino_get_matrix.argtypes = [vp, C.c_int, C.POINTER(_Rat), ip, ip]
    lib.wino_get_int_form.argtypes = [vp, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                      ip, ip]
    dp, sp = C.POINTER(ConvDesc), C.POINTER(Scales)
    lib.wino_workspace_bytes.argtypes = [dp, C.POINTER(C.c_size_t)]
    lib.wino_operand_bytes.argtypes = [dp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.wino_preferred_operand_layout.argtypes = [dp, ip]
    lib.wino_conv2d.argtypes = [dp, vp, vp, vp, sp, vp, C.c_size_t, vp]
    lib.wino_conv2d_noalloc.argtypes = [dp, vp, vp, vp, sp, vp]
    lib.wino_calibrate_workspace_bytes.argtypes = [dp, C.POINTER(C.c_size_t)]
    lib.wino_calibrate.argtypes = [dp, vp, vp, vp, sp, vp, C.c_size_t, vp]
    lib.wino_weight_transform.argtypes = [dp, vp, vp, sp, vp]
    lib.wino_input_transform.argtypes = [dp, vp, vp, sp, vp]
    lib.wino_transform_operands.argtypes = [dp, vp, vp, vp, vp, sp, vp]
    lib.wino_contract.argtypes = [dp, vp, vp, vp, sp, vp]
    lib.wino_output_transform.argtypes = [dp, vp, vp, sp, vp]
    lib.wino_contract_output.argtypes = [dp, vp, vp, vp, sp, vp]
    lib.wino_conv2d_launches.argtypes = [dp, C.c_char_p, C.c_size_t]
    lib.wino_set_option.argtypes = [C.c_int, C.c_int]
    fp = C.POINTER(FlexMatrices)
    lib.wino_flex_weight_transform.argtypes = [dp, fp, vp, vp, sp, vp]
    lib.wino_flex_input_transform.argtypes = [dp, fp, vp, vp, sp, vp]
    lib.wino_flex_output_transform.argtypes = [dp, fp, vp, vp, sp, vp]
    lib.wino_flex_conv2d.argtypes = [dp, fp, vp, vp, vp, sp, vp, C.c_size_t, vp]
    lib.wino_flex_calibrate.argtypes = [dp, fp, vp, vp, vp, sp, vp, C.c_size_t, vp]
    lib.wino_profile_next_launch.argtypes = [vp, vp]
    lib.wino_backward_workspace_bytes.argtypes = [dp, C.POINTER(C.c_size_t)]
    lib.wino_backward_dv_parts.argtypes = [dp, ip]
    lib.wino_backward.argtypes = [dp, vp, vp, vp, sp, vp, vp, vp, C.c_size_t, vp]
    lib.wino_flex_backward_workspace_bytes.argtypes = [dp, C.POINTER(C.c_size_t)]
    lib.wino_flex_backward.argtypes = [dp, fp, vp, vp, vp, vp, vp, vp, sp, vp, vp,
                                       C.POINTER(FlexGrads), vp, C.c_size_t, vp]
    lib.wino_probe_peak.argtypes = [C.c_int, C.c_int, C.c_int, vp, C.POINTER(C.c_double), vp]
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise WinoError(rc, _load().wino_last_error().decode())


class Matrices:
    """Exact rational matrices of one F(m, r) instance (host side)."""

    def __init__(self, m, r, mats, int_forms):
        self.m, self.r, self.n = m, r, m + r - 1
        self._mats, self._int = mats, int_forms
        for k, v in mats.items():
            setattr(self, k, v)

    def int_form(self, name):
        """(N, row_lcd) with matrix = diag(1/row_lcd) N."""
        return self._int[name]


def wino_make_matrices(m, r, points, base=BASE_LEGENDRE):
    """Exact Toom-Cook G, B^T, A^T and base-change factors; ``points`` are the
    m+r-2 finite points (ints or Fractions), infinity implicit and last."""
    lib = _load()
    pts = [Fraction(p) for p in points]
    arr = (_Rat * max(1, len(pts)))(*[_Rat(p.numerator, p.denominator) for p in pts])
    h = C.c_void_p()
    _check(lib.wino_make_matrices(m, r, arr, len(pts), base, C.byref(h)))
    try:
        mats, ints = {}, {}
        for which, name in enumerate(MAT_NAMES):
            buf = (_Rat * 64)()
            rows, cols = C.c_int(), C.c_int()
            _check(lib.wino_get_matrix(h, which, buf, C.byref(rows), C.byref(cols)))
            mats[name] = [[Fraction(buf[i * cols.value + j].num, buf[i * cols.value + j].den)
                           for j in range(cols.value)] for i in range(rows.value)]
            nb, lb = (C.c_int64 * 64)(), (C.c_int64 * 8)()
            _check(lib.wino_get_int_form(h, which, nb, lb, C.byref(rows), C.byref(cols)))
            ints[name] = ([[nb[i * cols.value + j] for j in range(cols.value)]
                           for i in range(rows.value)], [lb[i] for i in range(rows.value)])
    finally:
        lib.wino_free_matrices(h)
    return Matrices(m, r, mats, ints)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


def _scales(s):
    return s if isinstance(s, Scales) else Scales.from_dict(s)


def wino_profile_next_launch(start_event, stop_event):
    """Attach two raw hipEvent_t handles (ints) to the next kernel launch of this thread."""
    _check(_load().wino_profile_next_launch(C.c_void_p(start_event), C.c_void_p(stop_event)))


PROBE_MFMA_I8, PROBE_VALU_MAD24, PROBE_MFMA_BF16 = 0, 1, 2


def wino_probe_peak(kind, blocks, iters, sink, stream=None):
    """Launch one peak-probe kernel; returns the operations it performs."""
    work = C.c_double()
    _check(_load().wino_probe_peak(kind, blocks, iters, _ptr(sink), C.byref(work), _stream(stream)))
    return work.value


def wino_workspace_bytes(desc):
    out = C.c_size_t()
    _check(_load().wino_workspace_bytes(C.byref(desc), C.byref(out)))
    return out.value


def wino_backward_workspace_bytes(desc):
    out = C.c_size_t()
    _check(_load().wino_backward_workspace_bytes(C.byref(desc), C.byref(out)))
    return out.value


def wino_backward_dv_parts(desc):
    out = C.c_int()
    _check(_load().wino_backward_dv_parts(C.byref(desc), C.byref(out)))
    return out.value


def wino_backward(desc, dy, U, V, scales, dx, dw, workspace, stream=None):
    """Gradients of one layer w.r.t. its real input and weights (fp32); the
    workspace keeps dM, dU and dV."""
    sc = _scales(scales)
    _check(_load().wino_backward(C.byref(desc), _ptr(dy), _ptr(U), _ptr(V), C.byref(sc), _ptr(dx),
                                 _ptr(dw), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)))
    return dx, dw


def wino_flex_backward_workspace_bytes(desc):
    out = C.c_size_t()
    _check(_load().wino_flex_backward_workspace_bytes(C.byref(desc), C.byref(out)))
    return out.value


def wino_flex_backward(desc, fm, dy, x, w, U, V, M, scales, dx, dw, dGP, dBPT, dAPT, workspace,
                       stream=None):
    """Gradients of one flex layer: dx, dw and the gradients of the three trained
    matrices (device fp32 tensors dGP [n,3], dBPT [n,n], dAPT [m,n])."""
    sc = _scales(scales)
    grads = FlexGrads(dGP.data_ptr(), dBPT.data_ptr(), dAPT.data_ptr())
    _check(_load().wino_flex_backward(C.byref(desc), C.byref(fm), _ptr(dy), _ptr(x), _ptr(w),
                                      _ptr(U), _ptr(V), _ptr(M), C.byref(sc), _ptr(dx), _ptr(dw),
                                      C.byref(grads), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(),
                                      _stream(stream)))
    return dx, dw, dGP, dBPT, dAPT


def wino_calibrate_workspace_bytes(desc):
    out = C.c_size_t()
    _check(_load().wino_calibrate_workspace_bytes(C.byref(desc), C.byref(out)))
    return out.value


def wino_calibrate(desc, x, w, y, s_x, s_w, workspace, stream=None, per_point=False):
    """Device-side choice of every scale of a layer; returns a Scales struct.
    Runs the layer as a side effect (y may be None)."""
    sc = Scales.from_dict({"s_x": s_x, "s_w": s_w, "per_point": per_point})
    _check(_load().wino_calibrate(C.byref(desc), _ptr(x), _ptr(w), _ptr(y), C.byref(sc),
                                  _ptr(workspace), workspace.numel() * workspace.element_size(),
                                  _stream(stream)))
    return sc


def wino_conv2d(desc, x, w_or_V, y, scales, workspace, stream=None):
    """Whole layer on ``stream``; all tensors are caller-allocated device tensors."""
    sc = _scales(scales)
    _check(_load().wino_conv2d(C.byref(desc), _ptr(x), _ptr(w_or_V), _ptr(y), C.byref(sc),
                               _ptr(workspace), workspace.numel() * workspace.element_size(),
                               _stream(stream)))
    return y


NOALLOC_MAX_BYTES = 64 << 20


def wino_conv2d_noalloc(desc, x, w_or_V, y, scales, stream=None):
    """Whole layer with the library's built-in workspace (no allocation, no workspace argument);
    layers needing more than NOALLOC_MAX_BYTES of workspace are rejected."""
    sc = _scales(scales)
    _check(_load().wino_conv2d_noalloc(C.byref(desc), _ptr(x), _ptr(w_or_V), _ptr(y), C.byref(sc),
                                       _stream(stream)))
    return y


def wino_weight_transform(desc, w, V, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_weight_transform(C.byref(desc), _ptr(w), _ptr(V), C.byref(sc),
                                         _stream(stream)))
    return V


def wino_input_transform(desc, x, U, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_input_transform(C.byref(desc), _ptr(x), _ptr(U), C.byref(sc),
                                        _stream(stream)))
    return U


def wino_transform_operands(desc, x, U, w, V, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_transform_operands(C.byref(desc), _ptr(x), _ptr(U), _ptr(w), _ptr(V),
                                           C.byref(sc), _stream(stream)))
    return U, V


def wino_contract(desc, U, V, M, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_contract(C.byref(desc), _ptr(U), _ptr(V), _ptr(M), C.byref(sc),
                                 _stream(stream)))
    return M


def wino_output_transform(desc, M, y, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_output_transform(C.byref(desc), _ptr(M), _ptr(y), C.byref(sc),
                                         _stream(stream)))
    return y


def wino_operand_bytes(desc):
    """(bytes of V, bytes of U) in the order desc.operand_layout names."""
    v, u = C.c_size_t(), C.c_size_t()
    _check(_load().wino_operand_bytes(C.byref(desc), C.byref(v), C.byref(u)))
    return v.value, u.value


def wino_preferred_operand_layout(desc):
    """LAYOUT_* of a pretransformed V with which wino_conv2d runs this layer fastest."""
    out = C.c_int()
    _check(_load().wino_preferred_operand_layout(C.byref(desc), C.byref(out)))
    return out.value


def defragment(buf, n2, rows, channels):
    """A tensor in fragment order (flat int8 numpy array) back to [n2][rows][channels]:
    the inverse of the offset formula in include/wino.h, for tests and inspection."""
    import numpy as np
    rg, nch = -(-rows // 16), -(-channels // 64)
    a = np.asarray(buf).reshape(-1)[:n2 * rg * nch * 1024].reshape(n2, rg, nch, 4, 16, 16)
    # [p][row group][chunk][c%64/16][row%16][c%16] -> [p][row group][row%16][chunk][c%64/16][c%16]
    a = a.transpose(0, 1, 4, 2, 3, 5).reshape(n2, rg * 16, nch * 64)
    return a[:, :rows, :channels]


def wino_contract_output(desc, U, V, y, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_contract_output(C.byref(desc), _ptr(U), _ptr(V), _ptr(y), C.byref(sc),
                                        _stream(stream)))
    return y


OPT_AUTO_CONOUT = 1


def wino_set_option(option, value):
    _check(_load().wino_set_option(option, value))


def wino_conv2d_launches(desc):
    """Names of the kernel launches wino_conv2d makes for this descriptor, in order."""
    buf = C.create_string_buffer(128)
    _check(_load().wino_conv2d_launches(C.byref(desc), buf, 128))
    return [nm for nm in buf.value.decode().split(",") if nm]


def wino_flex_weight_transform(desc, fm, w, V, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_flex_weight_transform(C.byref(desc), C.byref(fm), _ptr(w), _ptr(V),
                                              C.byref(sc), _stream(stream)))
    return V


def wino_flex_input_transform(desc, fm, x, U, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_flex_input_transform(C.byref(desc), C.byref(fm), _ptr(x), _ptr(U),
                                             C.byref(sc), _stream(stream)))
    return U


def wino_flex_output_transform(desc, fm, M, y, scales, stream=None):
    sc = _scales(scales)
    _check(_load().wino_flex_output_transform(C.byref(desc), C.byref(fm), _ptr(M), _ptr(y),
                                              C.byref(sc), _stream(stream)))
    return y


def wino_flex_conv2d(desc, fm, x, w_or_V, y, scales, workspace, stream=None):
    """Whole layer with run-time fp32 matrices ``fm`` (a FlexMatrices)."""
    sc = _scales(scales)
    _check(_load().wino_flex_conv2d(C.byref(desc), C.byref(fm), _ptr(x), _ptr(w_or_V), _ptr(y),
                                    C.byref(sc), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(),
                                    _stream(stream)))
    return y


def wino_flex_calibrate(desc, fm, x, w, y, s_x, s_w, workspace, stream=None):
    """wino_calibrate for the flex layer; returns a Scales struct."""
    sc = Scales.from_dict({"s_x": s_x, "s_w": s_w})
    _check(_load().wino_flex_calibrate(C.byref(desc), C.byref(fm), _ptr(x), _ptr(w), _ptr(y),
                                       C.byref(sc), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(),
                                       _stream(stream)))
    return sc
