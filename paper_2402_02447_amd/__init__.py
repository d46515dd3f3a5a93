"""Bucket-wise gradient clipping fused with Adam for one MI355X (gfx950).

Thin ctypes binding over libbca.so (include/bca.h).  Every step of the path
runs in the library's HIP kernels; Python only marshals pointers and sizes.
"""
from .binding import (  # noqa: F401
    BCA_CLIP_WHOLE_GRADIENT, BCA_GRAD_BF16, BCA_GRAD_F16, BCA_GRAD_F32, BCA_SKIP_STEP_ON_NONFINITE, BCA_STATUS_BAD_THRESHOLD, BCA_STATUS_NONFINITE,
    BCA_TABLE_APPLY, BCA_TABLE_LAMB, BCA_TABLE_NORM, BCA_STATUS_TIMEOUT, BCA_STATUS_INCOMPLETE, BCA_TUNE_MULTI_LAUNCH, BCA_TUNE_STAGE_TABLE_LDS, BCA_TUNE_TICKETS, BCA_WRITE_BACK_GRADS, AdamHyper, BcaError, Plan, alg1_thresholds, bucket_clip_flat, copy_bytes, library_path, load_library, pack_device_hyper,
)
from .buckets import BucketLayout, flat_split, whole_tensors  # noqa: F401
