"""MI355X-native DETOX parameter-server step: thin Python binding over libdetox.so.

Every function here only marshals arguments (torch tensors -> device pointers, sizes, the
current HIP stream) into the C ABI declared in include/detox.h; all arithmetic runs in the
hand-written gfx950 kernels.  There is no CPU fallback: importing works without a GPU (so the
library's exports can be checked), calling anything needs one.
"""
from .binding import (  # noqa: F401
    AGG, DetoxError, OP, detox_block_mean, detox_filter_block_mean, detox_majority_filter,
    detox_sign_majority, detox_step, detox_step_robust_blocks, detox_step_static, lib, library_path, probe_mfma_f32, probe_stream_read, robust_bulyan, robust_coord_median,
    robust_coord_median_many, robust_geomedian, robust_geomedian_many,
    robust_blocks_workspace_bytes, robust_multikrum, robust_pairwise_sqdist, robust_trimmed_mean, strerror, trace, workspace_bytes)
