"""MI355X-native SageAttention forward pass: thin Python binding over the libsage C ABI.

The binding only marshals arguments (torch is used for device memory and streams); every step of
the path runs in the hand-written gfx950 kernels behind ``include/sage.h``.  There is no CPU
fallback: if the library is missing the import of :mod:`binding` raises.
"""
from .binding import (  # noqa: F401
    SageError,
    lib_path,
    load,
    sage_attn_cross_fwd,
    sage_attn_cross_split_fwd,
    sage_attn_fwd,
    sage_attn_pv_int8_cross_fwd,
    sage_attn_pv_int8_cross_split_fwd,
    sage_attn_pv_int8_fwd,
    sage_attn_clock_debug,
    sage_attn_qk_i32_debug,
    sage_attn_split_count,
    sage_attn_split_workspace,
    sage_default_sm_scale,
    sage_microbench,
    sage_quant_q,
    sage_quant_qk,
    sage_quant_v,
    sage_quant_v_pitch,
    sage_quant_v_workspace,
    sage_rope_quant_q,
    sage_rope_smooth_quant_k,
    sage_smooth_quant_k,
    NOALLOC_SCRATCH_BYTES,
    sage_smooth_quant_k_noalloc,
    sage_smooth_quant_k_workspace,
    sage_source_hash,
    sage_status_string,
    sageattn,
)
