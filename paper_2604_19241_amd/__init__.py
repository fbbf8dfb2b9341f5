"""MI355X-native fused MoE layer (routing, forward, backward) behind a C ABI.

The hot path lives in libuniep_moe.so (hand-written HIP for gfx950); this
package only marshals arguments.  See include/uniep_moe.h for the contract.
"""
from .binding import (  # noqa: F401
    GlobalMap, MoEError, MoEOpts, MoEShape, Routing, alloc_saved, load_library, make_opts,
    make_shape, moe_calibration_copy, moe_device_status, moe_fused_backward, moe_fused_forward,
    moe_global_map, moe_route, moe_route_backward, moe_route_static, alloc_routing,
    moe_calibration_mfma, ROUTE_STATIC_SCRATCH_BYTES, moe_saved_layout, moe_workspace_bytes, moe_backward_workspace_bytes,
    saved_views, status_string,
    MoEPerfConfig, MoEPerfHw, MoEPerfProblem, make_perf_hw, make_perf_problem,
    moe_perf_model_eval, moe_perf_model_search,
)
