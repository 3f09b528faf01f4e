"""MI355X-native forward pass of the Ternary-SVD linear map y = U (diag(S) (V x)).

Thin Python binding over the C-ABI library libtsvd.so (see include/tsvd.h).  The binding
only marshals arguments: every step of the computation runs in the HIP kernels.
"""
from .tsvd import (  # noqa: F401
    TSVD_F32, TSVD_BF16, TSVD_FEATURE_MAJOR, TSVD_TOKEN_MAJOR, TsvdError, Handle, lib_path, load_library,
    tsvd_dense_bytes, tsvd_dense_pack_host, tsvd_dense_unpack_host, tsvd_packed_bytes, tsvd_pack_host, tsvd_unpack_host, tsvd_pack, tsvd_unpack, tsvd_info,
    tsvd_workspace_bytes, tsvd_forward, tsvd_workspace_bytes_ex, tsvd_forward_ex, tsvd_forward_io, tsvd_forward_noalloc, TSVD_NOALLOC_MAX_WORKSPACE, tsvd_free, tsvd_strerror,
    tsvd_ternarize, tsvd_fit_scales, tsvd_residual, tsvd_leading_singular_pair, tsvd_transition,
    tsvd_conv2d_forward,
    tsvd_tuning_set, tsvd_tuning_reset, tsvd_tuning_forward_stages, tsvd_tuning_tile_shapes, tsvd_tuning_read_clocks,
)
