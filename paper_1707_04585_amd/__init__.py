"""MI355X-native reversible residual block library (thin Python binding).

All computation happens in the HIP library ``librevnet_hip.so`` behind the C
ABI of ``include/revnet.h``; this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    BASIC, BOTTLENECK, BF16, F32, BlockDesc, RevnetError, lib_path, load_library, pack_grads,
    pack_params, revnet_block_bwd_reconstruct, revnet_block_fwd, revnet_last_error, revnet_profile_begin, revnet_profile_end,
    revnet_stack_bwd, revnet_stack_cost, revnet_stack_fwd, revnet_version, revnet_workspace_bytes,
    BodyDesc, DownDesc, pack_down, pack_stages, revnet_body_bwd, revnet_body_fwd, revnet_body_workspace_bytes,
    revnet_down_bwd, revnet_down_fwd, revnet_down_workspace_bytes,
    revnet_fixed_from_float, revnet_fixed_to_float, revnet_fixed_workspace_bytes, revnet_stack_bwd_fixed,
    revnet_stack_fwd_fixed, revnet_stem_bwd, revnet_stem_fwd, revnet_stem_workspace_bytes, rvn_stem_desc,
    revnet_body_bwd_fixed, revnet_body_fixed_workspace_bytes, revnet_body_fwd_fixed,
    revnet_stack_fwd_static, STATIC_WS_BYTES,
)
