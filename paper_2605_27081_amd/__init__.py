"""MI355X-native MoE-layer hot path and routing-trace statistics (thin binding over the C ABI).

Every step runs in the HIP library `libremoe_hip.so` (sources in csrc/, declarations in
include/remoe.h); this package only marshals arguments.  There is no CPU fallback: calls fail
loudly when the library has not been built.
"""
from .binding import (  # noqa: F401
    LayerDesc,
    REMOE_CACHE_BELADY,
    REMOE_CACHE_FIFO,
    REMOE_CACHE_LFU,
    REMOE_CACHE_LRU,
    cache_simulate,
    remoe_cache_workspace_bytes,
    reroute_lru,
    routing_balance,
    step_miss_summary,
    REMOE_DECODE_CHAINED,
    REMOE_DECODE_PIPELINED,
    RemoeError,
    library_path,
    load_library,
    lru_simulate,
    moe_decode,
    moe_decode_static,
    remoe_copy_probe,
    remoe_decode_workspace_bytes,
    remoe_decode_static_bytes,
    moe_forward,
    moe_route,
    PROF_KINDS,
    remoe_last_error,
    remoe_gate_grad,
    remoe_gate_grad_workspace_bytes,
    remoe_loss_backward,
    remoe_loss_backward_workspace_bytes,
    remoe_loss_forward,
    remoe_loss_workspace_bytes,
    remoe_profile_enable,
    remoe_profile_read,
    remoe_version,
    remoe_workspace_bytes,
    trace_reuse,
)
