"""MI355X (gfx950) ternary 3D convolution: thin Python binding over the C ABI in include/tern.h.

The binding marshals arguments only; every step of the path (packing, convolution, activation,
re-packing) runs in the HIP kernels of libtern.so.  PyTorch is used for device memory and streams.
There is no CPU fallback: importing works without a GPU (so that the library can be built and its
symbols checked), but every compute call needs the built library and a device tensor.
"""
from .binding import (  # noqa: F401
    TernError,
    lib,
    lib_path,
    tern_concat,
    tern_conv3d,
    tern_conv3d_binary,
    tern_pack_filters_binary,
    tern_binary_bank_bytes,
    tern_count_codes,
    tern_conv3d_real,
    tern_fold_avgpool,
    tern_pool_digits,
    tern_digits_weights,
    tern_conv_out_dims,
    tern_fcn_forward,
    tern_net_forward,
    tern_net_workspace_bytes,
    NetModule,
    tern_fcn_workspace_bytes,
    tern_static_scratch_bytes,
    tern_filter_bank_bytes,
    tern_matrix_bank_bytes,
    tern_expand_filters,
    tern_fold_batchnorm,
    tern_fold_thresholds,
    tern_ternarize_filters,
    tern_ternarize_filters_sparse,
    tern_pack,
    tern_pack_filters,
    tern_packed_bytes,
    tern_probe_valu,
    tern_set_option,
    tern_threshold_pack,
    tern_words,
    FcnLayer,
)
