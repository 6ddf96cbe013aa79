"""MI355X-native GR-KAN group-wise rational function (FlashKAT hot path).

The product is libgrkan.so (hand-written HIP for gfx950 behind the C ABI in
include/grkan.h); this package is its thin Python binding.
"""
from .binding import (  # noqa: F401
    DEGREES,
    GRKAN_BF16,
    GRKAN_F16,
    GRKAN_F32,
    GrkanError,
    Plan,
    device_query,
    grkan_alg1_bwd,
    grkan_bwd,
    grkan_bwd_noalloc,
    grkan_bwd_raw,
    grkan_bwd_workspace_bytes,
    grkan_fwd,
    PackedWeight,
    grkan_linear_fwd,
    grkan_linear_pack_w,
    grkan_fwd_raw,
    load_library,
    plan,
    plan_cover_errors,
    status_string,
    tuning_override,
)
