"""MI355X-native fused attention for LLM inference (prefill, chunked prefill, paged decode).

Thin ctypes binding over ``libattn_gfx950.so``; every step of the computation runs in the
library's HIP kernels.  PyTorch tensors only provide device memory and streams.
"""
from .binding import (  # noqa: F401
    ATTN_BF16,
    ATTN_F16,
    ATTN_F32,
    AttnArgs,
    AttnError,
    attn_clear_cache,
    attn_decode_paged,
    attn_environment_key,
    attn_force_instance,
    attn_instance_name,
    attn_load_cache,
    attn_num_instances,
    attn_prefill_varlen,
    attn_selected_instance,
    attn_status_string,
    attn_tune,
    attn_workspace_bytes,
    library_path,
    load_library,
    make_args,
    KvWriteArgs,
    attn_kv_cache_write,
    make_kv_write_args,
    RmsNormArgs,
    make_rmsnorm_args,
    rmsnorm_force_instance,
    rmsnorm_fused_add,
    rmsnorm_instance_name,
    rmsnorm_num_instances,
    rmsnorm_selected_instance,
    rmsnorm_tune,
)
