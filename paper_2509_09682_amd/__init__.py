"""MI355X-native fused cross-entropy with negative sampling (CCE-): HIP kernels behind a C ABI, plus a ctypes binding."""
from .binding import (  # noqa: F401
    CCE_ALGO_AUTO, CCE_ALGO_GATHER, CCE_ALGO_TILE, CCE_BF16, CCE_F32, CCE_NEG_FULL, CCE_NEG_PER_POSITION,
    CCE_NEG_SHARED, CCE_OK, CCE_ERR_NULL, CCE_ERR_SHAPE, CCE_ERR_DTYPE, CCE_ERR_INDEX, CCE_ERR_WORKSPACE, CCE_ERR_UNSUPPORTED,
    CCE_ERR_HIP, CceDesc, CceError, cce_neg_backward, cce_neg_forward, cce_neg_forward_noalloc, cce_neg_index_status,
    CCE_SAMPLER_ALIAS, CCE_SAMPLER_UNIFORM, CceSampler, cce_neg_backward_sampled, cce_neg_forward_sampled, cce_neg_sample,
    make_sampler, cce_neg_workspace_bytes, cce_neg_workspace_init, cce_neg_profile_enable, cce_neg_profile_read, make_desc, new_workspace, status_string,
)
from .autograd import cce_neg_loss, clear_workspaces  # noqa: F401,E402
from .consumers import bucketed_step  # noqa: F401,E402
