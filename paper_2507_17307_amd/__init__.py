"""MI355X-native hot path of entropy-routed stitched decoding.

The product is ``librstitch.so`` (HIP kernels for gfx950 behind a C ABI, see
``include/rstitch.h``); this package is its thin Python binding.  There is no
CPU fallback: importing the binding without the built library raises.
"""

from .binding import (  # noqa: F401
    RS_SLM, RS_LLM, FLAG_HI, FLAG_ACCEPT, FLAG_NEXT_LLM, FLAG_NONFINITE, FLAG_BADARG, FLAG_ABORTED, FLAG_ROUTER_STAY,
    RsError, RsConfig, RouteOut, lib, library_path,
    rs_abi_version, rs_last_error, rs_workspace_bytes, rs_kv_bytes, rs_create_model, rs_destroy_model,
    rs_decode_step, rs_catchup_prefill, rs_route, rs_route_plus, RouterPlus, rs_route_static, rs_route_scratch_bytes, rs_set_phase_timer, rs_set_spin_limit, rs_set_sampling,
    rs_stitch_generate, STITCH_RUNNING, STITCH_DONE, STITCH_TRACE_FULL, STITCH_FLAGGED, STITCH_ABORTED,
    Model,
)
