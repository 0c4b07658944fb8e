"""MI355X-native APOLLO / APOLLO-Mini optimizer step (arXiv 2412.05270, Algorithm 1), and the
element-wise AdamW (Section 3.1) for the parameters APOLLO does not project.

Thin ctypes binding over the C-ABI library built from csrc/ (see include/apollo.h for the
contract of every call).  Everything numerical happens in the HIP kernels; this package only
marshals arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    APOLLO_BF16, APOLLO_CHANNEL, APOLLO_DBG_C, APOLLO_DBG_COLSQ, APOLLO_DBG_M, APOLLO_DBG_NORM,
    APOLLO_DBG_R, APOLLO_DBG_S, APOLLO_DBG_V, APOLLO_EHIP, APOLLO_EINVAL, APOLLO_ENOMEM, APOLLO_ESTATE,
    APOLLO_EUNSUPPORTED, APOLLO_F32, APOLLO_OK, APOLLO_PATH_GENERAL, APOLLO_PATH_MATRIX_CORE,
    APOLLO_PATH_NONE, APOLLO_PATH_RANK1, APOLLO_PROJ_IDENTITY, APOLLO_PROJ_RANDOM, APOLLO_Q8,
    APOLLO_ROUND_NEAREST, APOLLO_ROUND_STOCHASTIC, APOLLO_SCHEDULE_OVERLAP, APOLLO_SCHEDULE_CHUNKED, APOLLO_SCHEDULE_SERIAL,
    APOLLO_SIDE_AUTO, APOLLO_SIDE_LEFT, APOLLO_SIDE_RIGHT, APOLLO_TENSOR,
    AdamwStepper, ApolloAdamwConfig, ApolloConfig, ApolloError, ApolloFlatShape, ApolloShape,
    ApolloStepper, ApolloTensor,
    apollo_adamw_destroy, apollo_adamw_init, apollo_adamw_last_error, apollo_adamw_state_bytes,
    apollo_adamw_state_offsets, apollo_adamw_step, apollo_adamw_workspace_bytes, apollo_debug_copy,
    apollo_debug_fill_projection, apollo_debug_gauss_parts, apollo_debug_get, apollo_debug_path,
    apollo_debug_philox, apollo_destroy, apollo_init, apollo_last_error, apollo_profile_enable,
    apollo_profile_read, apollo_state_bytes, apollo_state_offsets, apollo_step, apollo_step_launch, apollo_step_noalloc, apollo_step_prepare,
    apollo_workspace_bytes, APOLLO_NOALLOC_MAX_TENSORS, APOLLO_NOALLOC_SCRATCH_BYTES,
    library_path, load_library)
