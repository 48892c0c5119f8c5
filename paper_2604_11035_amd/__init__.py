"""MI355X (gfx950) hot path of one introspective-strided-decoding step.

Thin Python binding over the C ABI declared in include/idlm.h: the functions here
only marshal arguments (device pointers, sizes, the current HIP stream); every
step of the path runs in the hand-written HIP kernels of libidlm_isd.so.  There
is no CPU or PyTorch fallback: if the library is missing, importing the binding
functions raises.
"""
from .binding import (IdlmError, idlm_gated_lora_linear, idlm_gated_lora_linear_workspace, idlm_isd_accept, idlm_isd_accept_bf16, idlm_isd_accept_workspace,
                      idlm_isd_accept_static, idlm_isd_accept_static_max_bytes,
                      idlm_isd_accept_filtered, idlm_isd_accept_filtered_q, idlm_isd_accept_filtered_workspace,
                      idlm_isd_accept_general, idlm_isd_accept_general_workspace,
                      idlm_isd_attention, idlm_isd_commit, idlm_isd_rng_dump, idlm_isd_kv_append, idlm_isd_validate,
                      idlm_isd_attention_workspace, idlm_stream_copy,
                      idlm_isd_attention_wave_trace, idlm_stream_read, idlm_strerror, idlm_version, lib, lib_path)

__all__ = [
    "IdlmError", "idlm_gated_lora_linear", "idlm_gated_lora_linear_workspace", "idlm_isd_accept", "idlm_isd_accept_bf16", "idlm_isd_accept_workspace", "idlm_isd_accept_static", "idlm_isd_accept_static_max_bytes", "idlm_isd_attention",
    "idlm_isd_commit", "idlm_isd_rng_dump", "idlm_isd_kv_append", "idlm_isd_validate", "idlm_isd_accept_general", "idlm_isd_accept_general_workspace",
    "idlm_isd_accept_filtered", "idlm_isd_accept_filtered_q", "idlm_isd_accept_filtered_workspace",
    "idlm_isd_attention_workspace", "idlm_stream_copy",
    "idlm_isd_attention_wave_trace", "idlm_stream_read", "idlm_strerror", "idlm_version", "lib", "lib_path",
]
