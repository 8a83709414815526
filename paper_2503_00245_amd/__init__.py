"""MI355X-native sparse MoE feed-forward layer (CoSMoEs, arXiv 2503.00245): HIP kernels for
gfx950 behind the C ABI of include/moe.h, plus a ctypes binding of the same names."""
from .binding import (  # noqa: F401
    EXPORTS, FLAG_RESIDUAL, FLAG_SHARED_BASE, LIB_PATH, MOE_BF16, MOE_F32, MoeError, MoeShape,
    MoeWeights, alloc_workspace, lib, make_shape, make_weights, moe_combine, moe_expert_ffn,
    moe_bles_loss, moe_bles_workspace_bytes, moe_delta_uniform, moe_expert_replacements, moe_forward,
    moe_forward_static, moe_forward_timed, STATIC_WORKSPACE_BYTES, moe_offload_counters, moe_permute, moe_route, moe_stack_forward, moe_workspace_bytes, shape_for,
    status_string,
)
