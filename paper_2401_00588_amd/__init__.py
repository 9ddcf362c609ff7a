"""MI355X-native hot path of one Virtual Token Counter serving step.

Thin Python binding over the C ABI of ``include/vtc.h``: argument marshalling
only -- every step of the path runs in the HIP kernels of ``libvtc_mi355x.so``.
There is no CPU fallback: calling any entry point without the built library
raises.
"""
from .binding import (  # noqa: F401
    AttnParams,
    CostPoly,
    HipEvent,
    VTC_BF16,
    VTC_F16,
    VTC_F32,
    VtcError,
    library_path,
    load_library,
    make_params,
    vtc_attn_decode,
    vtc_attn_decode_static,
    vtc_attn_prefill_chunk,
    vtc_attn_workspace_bytes,
    vtc_counter_update,
    vtc_counter_update_cost,
    vtc_counter_update_predicted,
    vtc_kv_append,
    vtc_step_decode,
    vtc_debug_gather_slots,
    vtc_strerror,
    vtc_version,
)
