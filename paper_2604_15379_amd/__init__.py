"""MI355X-native decode-step megakernel (persistent task-graph HIP kernel).

The package is a thin ctypes binding over ``libfleet.so`` (C ABI declared in
``include/fleet.h``); every step of the decode path runs in the HIP kernels.
"""
from .binding import (  # noqa: F401
    FleetError, Fleet, SCHED_COOPERATIVE, SCHED_UNAWARE, SCHED_MSPLIT, FLAG_TRACE, FLAG_SINGLE_LEVEL,
    FLAG_NO_SPLITK, FLAG_NO_STREAM, FLAG_NO_RESIDENT, FLAG_UNFUSED_SILU,
    FLAG_SEPARATE_NORM, FLAG_CHAINED, FLAG_TIMING, FLAG_PACKED_ONLY, FLAG_NT_STORES, STATIC_SCRATCH_BYTES,
    fleet_decode_step_static, fleet_create, fleet_decode_step, fleet_decode_layers, fleet_decode_tokens, fleet_decode_step_paged, fleet_destroy,
    fleet_gemm, fleet_graph_build, fleet_graph_dump, fleet_trace_read, fleet_last_status,
    fleet_device_probe, fleet_copy, fleet_weight_bytes, fleet_weight_bytes_per_xcd, fleet_l2_window_bytes,
    fleet_l2_hit_model, fleet_effective_intensity, fleet_step_bytes, fleet_strerror,
    load_library, parse_graph, EXPORTS,
)
