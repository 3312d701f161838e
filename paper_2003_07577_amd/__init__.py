"""MI355X-native mixed-precision convolution by binary decomposition.

Thin Python binding over the C-ABI library ``libebs.so`` (see ``include/ebs.h``).
The binding only marshals arguments; every step runs in the library's HIP
kernels.  PyTorch is used by callers for device memory and streams only.
"""
from .binding import (  # noqa: F401
    EbsError,
    ebs_check_levels,
    ebs_conv_variant_count,
    ebs_conv_variant_name,
    ebs_mixed_conv2d,
    ebs_mixed_conv2d_mfma_i8,
    ebs_mixed_conv2d_requant,
    ebs_mixed_conv2d_signed,
    ebs_partial_products_bytes,
    ebs_quantize_weights,
    ebs_quantize_weights_static,
    STATIC_MAX_COUNT,
    ebs_quantize_activations,
    ebs_aggregate_weights,
    ebs_aggregate_activations,
    QUANT_WORKSPACE_BYTES,
    MAX_CANDIDATES,
    ebs_binary_conv_planes,
    ebs_pow2_depthwise,
    ebs_mixed_conv2d_variant,
    ebs_pack_activations,
    ebs_pack_weights,
    ebs_probe_and_bcnt,
    ebs_probe_and_bcnt_pairs,
    ebs_probe_copy,
    ebs_packed_activations_bytes,
    ebs_packed_weights_bytes,
    ebs_status_string,
    ebs_last_hip_error,
    ebs_version,
    library_path,
    load_library,
    out_dims,
)
