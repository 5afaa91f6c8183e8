"""MI355X-native HQMQ KV-cache encode / decode.

The product is the C-ABI library ``libhqmq.so`` (HIP kernels for gfx950, declared in
``include/hqmq.h``); this package is its thin Python binding: the functions below have the
library's names and only marshal arguments.  PyTorch provides device memory and streams.
"""
from .binding import (  # noqa: F401
    HQMQ_FLAG_CHECK_FINITE,
    HQMQ_FLAG_NO_OUTLIERS,
    HQMQ_MAX_S,
    HQMQ_STATIC_SCRATCH_BYTES,
    HQMQ_STATUS_NONFINITE,
    HQMQ_STATUS_OUTLIER_OVERFLOW,
    DecodeBatch,
    EncodeBatch,
    EncodedBuffers,
    HqmqError,
    HqmqParams,
    HqmqSizeInfo,
    alloc_batch_workspace,
    alloc_encoded,
    alloc_workspace,
    hqmq_attend,
    hqmq_attend_lse,
    hqmq_attend_masked,
    hqmq_attend_workspace_bytes,
    hqmq_build_codebooks,
    hqmq_decode,
    hqmq_decode_batch,
    hqmq_encode,
    hqmq_encode_batch,
    hqmq_encode_batch_given_thresholds,
    hqmq_encode_given_thresholds,
    hqmq_encode_static,
    hqmq_encode_timed,
    hqmq_init,
    hqmq_last_hip_error,
    hqmq_shard_median_pass,
    hqmq_shard_median_region,
    hqmq_sizes,
    hqmq_thresholds,
    library_path,
    params_for,
)
