"""MI355X-native quantised Winograd convolution in the Legendre base.

Thin ctypes binding over libwino.so (HIP kernels + C ABI, see include/wino.h).
PyTorch is used for device memory and streams only; every step of the
convolution runs in the library's kernels.  Importing this package without a
built library raises: there is no CPU fallback.
"""
from .binding import (  # noqa: F401
    BASE_CANONICAL, BASE_CHEBYSHEV, BASE_HERMITE, BASE_LEGENDRE, FUSED_AUTO, FUSED_OFF, FUSED_ON,
    OUT_F32, OUT_I32, OUT_I8, MAT_NAMES, PROBE_MFMA_BF16, PROBE_MFMA_I8, PROBE_VALU_MAD24, ConvDesc, FlexGrads, FlexMatrices, Matrices, Scales, WinoError,
    lib_path, wino_backward, wino_backward_dv_parts, wino_backward_workspace_bytes, wino_calibrate,
    wino_calibrate_workspace_bytes, wino_contract, wino_contract_output, wino_conv2d, wino_conv2d_noalloc, NOALLOC_MAX_BYTES,
    wino_conv2d_launches, wino_set_option, wino_operand_bytes, wino_preferred_operand_layout, defragment, OPT_AUTO_CONOUT,
    LAYOUT_FRAGMENTS, LAYOUT_ROWS,
    wino_flex_backward, wino_flex_backward_workspace_bytes, wino_flex_calibrate, wino_flex_conv2d, wino_flex_input_transform,
    wino_flex_output_transform, wino_flex_weight_transform, wino_input_transform,
    wino_make_matrices, wino_output_transform, wino_probe_peak, wino_profile_next_launch,
    wino_transform_operands, wino_weight_transform, wino_workspace_bytes,
)
