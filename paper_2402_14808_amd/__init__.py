"""MI355X (gfx950) relay attention: hand-written HIP kernels behind a C ABI
(include/relay_attn.h) and a thin ctypes binding with the same names."""
from .binding import (RADecodePlan, RAParams, RAPrefix, RAValidateReport, RelayAttnError, load,
                      make_params, make_prefixes, paged_attn_decode_naive,
                      relay_attn_cache_append, relay_attn_debug_decode_phases,
                      relay_attn_debug_launch_probe, relay_attn_debug_stream_probe,
                      relay_attn_debug_timeline,
                      relay_attn_debug_validate, relay_attn_decode, relay_attn_decode_append,
                      relay_attn_decode_grouped, relay_attn_group_requests,
                      relay_attn_decode_multi, relay_attn_decode_plan, relay_attn_decode_static,
                      relay_attn_prefill, relay_attn_prefill_multi, relay_attn_static_scratch_bytes,
                      relay_attn_system_cache_layout, relay_attn_system_fill,
                      relay_attn_workspace_bytes, status_string, system_cache_view)

__all__ = ["RADecodePlan", "RAParams", "RAPrefix", "RAValidateReport", "RelayAttnError", "load",
           "make_params", "make_prefixes", "paged_attn_decode_naive", "relay_attn_cache_append",
           "relay_attn_debug_decode_phases", "relay_attn_debug_launch_probe",
           "relay_attn_debug_stream_probe", "relay_attn_debug_timeline", "relay_attn_debug_validate", "relay_attn_decode",
           "relay_attn_decode_append", "relay_attn_decode_grouped", "relay_attn_group_requests",
           "relay_attn_decode_multi", "relay_attn_decode_plan",
           "relay_attn_decode_static", "relay_attn_static_scratch_bytes",
           "relay_attn_prefill", "relay_attn_prefill_multi", "relay_attn_system_cache_layout",
           "relay_attn_system_fill", "relay_attn_workspace_bytes", "status_string", "system_cache_view"]
