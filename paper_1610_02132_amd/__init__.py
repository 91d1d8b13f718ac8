"""MI355X-native QSGD hot path: thin Python binding over libqsgd.so (HIP, gfx950).

Every step of Encode / Decode / step runs in the library's kernels; this package
only marshals arguments (device pointers of torch tensors, the current HIP
stream).  There is no CPU fallback: importing the binding fails if the library
has not been built (``python -m paper_1610_02132_amd.build``).
"""
from .binding import (  # noqa: F401
    CODE_DENSE, CODE_FIXED, CODE_SPARSE, NORM_L2, NORM_MAX, QSGD_MAX_PEERS, Params, QsgdError,
    lib_path, qsgd_decode_accumulate, qsgd_encode, qsgd_max_encoded_bytes, qsgd_message_info,
    qsgd_copy_probe, qsgd_message_status, qsgd_sgd_step, qsgd_strerror, qsgd_timing_enable, qsgd_timing_get,
    qsgd_timing_reset, qsgd_version, qsgd_workspace_bytes, qsgd_workspace_status,
    Layout, qsgd_decode_accumulate_layout, qsgd_encode_layout, qsgd_layout_info,
    qsgd_layout_max_encoded_bytes, qsgd_layout_workspace_bytes, qsgd_sgd_step_layout,
    Pipeline, qsgd_encode_slice, qsgd_pipeline_step, qsgd_copy_probe_words,
    qsgd_encode_workspace_bytes, qsgd_encode_static, qsgd_static_scratch_bytes,
)
