"""MI355X-native quantized-inference hot path (arXiv 1806.08342): thin Python binding over
the C-ABI library ``libqnn.so`` built from the HIP sources in ``csrc/``.

PyTorch is used for device memory and streams only; every step of the path runs in the
library's own kernels.  Importing the package does not load the library; the first call
does, and fails loudly when it has not been built.
"""
from .binding import (  # noqa: F401
    calibrate_copy,
    calibrate_mfma,
    calibrate_rescale,
    QnnError,
    act_range,
    choose_qparams,
    dequantize,
    library_path,
    load_library,
    minmax,
    new_range_state,
    pack_b,
    pack_int4,
    prepare_qgemm,
    qadd,
    qadd_params,
    qconv2d,
    qconv2d_add,
    qconv2d_asym,
    qconv2d_workspace_bytes,
    qdwconv2d,
    qdwconv2d_asym,
    qgemm,
    qgemm_add,
    qgemm_asym,
    qgemm_noalloc,
    qgemm_plan,
    qgemm_workspace_bytes,
    quantize,
    quantize_dynamic,
    quantize_with,
    read_range_state,
    quantize_u16,
    dequantize_u16,
    simquant,
    simquant_backward,
    quantize_multiplier,
    quantize_multipliers,
    quantize_weights,
    requantize,
    rescale_u8,
    tuning_set,
)

__all__ = [
    "QnnError", "act_range", "choose_qparams", "dequantize", "library_path", "load_library", "minmax", "new_range_state", "pack_b", "pack_int4", "prepare_qgemm",
    "qadd", "qadd_params", "qconv2d", "qconv2d_add", "qconv2d_asym", "qdwconv2d", "qdwconv2d_asym", "qgemm", "qgemm_add", "qgemm_asym", "qgemm_plan", "quantize", "quantize_dynamic", "quantize_with", "read_range_state", "quantize_u16", "dequantize_u16", "simquant", "simquant_backward", "quantize_multiplier",
    "quantize_multipliers", "quantize_weights", "requantize", "rescale_u8", "qgemm_workspace_bytes", "qconv2d_workspace_bytes", "tuning_set", "calibrate_copy", "calibrate_mfma", "calibrate_rescale", "qgemm_noalloc",
]
