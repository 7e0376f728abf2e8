"""MI355X-native runtime hot path of Pairwise Rotation Quantization (arXiv 2511.10645).

Thin Python binding over the C ABI of ``libparo.so`` (``include/paro.h``): argument
marshalling only.  Every step of the path runs in the library's HIP kernels; PyTorch is used
for device memory and streams.  There is no CPU fallback: a missing library is an error.
"""
from .binding import (  # noqa: F401
    ParoError,
    paro_diag_mfma_f16,
    paro_diag_read_stream,
    paro_fwht,
    Rotation,
    W4Weight,
    lib,
    lib_path,
    paro_rotate_scale,
    paro_rotate_scale_quantize_int4,
    paro_rotate_scale_quantize_mxfp4,
    paro_rotated_linear,
    paro_rotated_linear_multi,
    paro_rotated_linear_noalloc,
    paro_rotation_plan_build,
    paro_select_pairs_host,
    paro_status_string,
    paro_validate_pairs_host,
    paro_version,
    paro_w4_dequant,
    paro_w4_quantize,
    paro_w4_repack,
    paro_w4_unpack_codes,
    paro_w4_unpack_zeros,
    paro_w4a16_linear,
    paro_workspace_bytes,
    paro_workspace_exchange_bytes,
    paro_workspace_exchange_bytes_multi,
    paro_workspace_bytes_multi,
    Workspace,
)
