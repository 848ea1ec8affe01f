"""MI355X (gfx950) Cross-Self Pruning: thin Python binding over libcsp.so.

All computation happens in the HIP kernels behind the C ABI declared in
include/csp.h; this package only marshals torch tensors (device memory and
streams) into that ABI.  There is no CPU fallback: if libcsp.so has not been
built the first call raises.
"""
from .binding import (  # noqa: F401
    CspError, Desc, lib_path, load_library,
    csp_score, csp_score_lse, csp_select, csp_compact, csp_decode_attn, csp_decode_attn_static, csp_static_scratch_bytes, csp_decode_step, csp_decode_step_phase, csp_append_kv,
    csp_gather_modality, csp_window_push, csp_decode_step_window, csp_reprune, csp_probe_stream,
    csp_score_workspace_bytes, csp_select_workspace_bytes, csp_decode_workspace_bytes, csp_reprune_workspace_bytes,
    csp_strerror, csp_version, EXPORTED_SYMBOLS,
)
