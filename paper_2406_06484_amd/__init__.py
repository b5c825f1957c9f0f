"""MI355X-native chunkwise-parallel DeltaNet forward/backward (hand-written HIP behind a C ABI).

``deltanet_fwd`` / ``deltanet_bwd`` / ``deltanet_recurrent_fwd`` are thin argument-marshalling bindings over
``libdeltanet_hip.so`` (see ``include/deltanet.h``).  There is no CPU or PyTorch fallback: if the
library has not been built, calling them raises.
"""
from .binding import (  # noqa: F401
    DN_OPT_STREAMED_CHUNK_KERNEL,
    DeltaNetError,
    deltanet_bwd,
    deltanet_bwd_saved,
    deltanet_fused_bwd,
    deltanet_fused_bwd_saved,
    deltanet_fused_fwd,
    deltanet_fused_fwd_save,
    deltanet_fused_workspace_bytes,
    deltanet_fwd,
    deltanet_fwd_save,
    deltanet_fwd_static,
    deltanet_gated_bwd,
    deltanet_gated_bwd_saved,
    deltanet_gated_fwd,
    deltanet_gated_fwd_save,
    deltanet_gated_recurrent_fwd,
    deltanet_gated_workspace_bytes,
    deltanet_lds_probe,
    deltanet_profile_collect,
    deltanet_recurrent_fwd,
    deltanet_set_option,
    deltanet_profile_enable,
    deltanet_status_string,
    deltanet_workspace_bytes,
    library_path,
    load_library,
)
