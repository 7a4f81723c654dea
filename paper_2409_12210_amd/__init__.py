"""MI355X (gfx950) implementation of one Mixture-of-Diverse-Size-Experts FFN layer
(arXiv 2409.12210).  All computation runs in hand-written HIP kernels behind the C ABI declared in
include/modse.h; this package only marshals arguments.  There is no CPU fallback: calls raise if the
compiled library is missing."""
from .binding import (  # noqa: F401
    STAGES, WS_BWD, WS_FWD, WS_FWD_SAVED, GateExt, ModseError, Routing, lib_path, load_library, modse_layer_bwd, modse_layer_bwd_ext,
    modse_layer_fwd, modse_layer_fwd_ext, modse_route, modse_route_ext, modse_route_static, modse_routing_stats,
    modse_saved_size,
    modse_stage_times, modse_stage_timing_enable, modse_status_string, modse_workspace_size,
)
