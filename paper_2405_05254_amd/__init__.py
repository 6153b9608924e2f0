"""libyoco: YOCO's attention hot path on MI355X, behind a C ABI.

The Python layer only marshals arguments (torch tensors -> device pointers,
the current HIP stream); every step of the path runs in the HIP kernels of
libyoco.so. There is no CPU fallback: a missing library raises.
"""
from .binding import (  # noqa: F401
    F32, BF16, INT8, YocoError, KVCache, lib, lib_path,
    kv_cache_bytes, swa_prefill, global_kv_write, global_kv_write_scaled, cross_attn_prefill,
    cross_attn_decode, cross_attn_decode_workspace, cross_attn_decode_noalloc, NOALLOC_SCRATCH_BYTES, version,
    swa_cache_write, kv_cache_append, swa_decode,
    gret_prefill_workspace, gret_prefill, gret_decode, ceiling_mfma, ceiling_attn_loop, ceiling_stream_read,
)
