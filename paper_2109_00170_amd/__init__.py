"""MI355X-native SIMD-structured sparse convolution (hot path of arXiv 2109.00170, Section 3.2).

Thin ctypes binding over ``libalcs.so`` (see ``include/alcs.h``); every step of the
path runs in the HIP library.  There is no CPU fallback: if the library has not been
built, loading fails with an ImportError.
"""
from ._binding import (  # noqa: F401
    AlcsError,
    HipEvents,
    Options,
    Packed,
    alcs_block_scores,
    alcs_dense_conv,
    alcs_depthwise_conv,
    alcs_dw_sparse_conv_fused,
    alcs_last_launch,
    alcs_latency_estimate,
    alcs_network_latency,
    alcs_pack_csr_device,
    alcs_pack_from_csr,
    alcs_pack_from_csr_device,
    alcs_pack_network_device,
    alcs_pack_workspace_bytes,
    alcs_pack_weights_device,
    alcs_pack_on_device,
    alcs_pack_weights,
    alcs_project_latency,
    alcs_sparse_conv,
    alcs_sparse_conv_bf16,
    alcs_sparse_conv_bf16_mfma,
    alcs_sparse_conv_fused,
    alcs_strerror,
    alcs_topn_mask,
    alcs_topn_mask_static,
    alcs_version,
    library_path,
    load_library,
    out_size,
)
