"""fp64 CPU oracle for the YOCO attention hot path.

TEST INFRASTRUCTURE ONLY. Nothing in the product package may import this
package; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg
use it. It shares no code with the HIP path.
"""
from .yoco_oracle import (  # noqa: F401
    swa_row, swa, rmsnorm, global_kv, global_kv_scaled_form, cross_attn_row, cross_attn,
    swish, swiglu, yoco_stack, kv_cache_bytes_per_token, RollingWindowCache, yoco_stack_generate,
    gret_decay, gret_parallel, gret_recurrent, gret_chunkwise, group_norm_heads, mhgr,
    kv_quantise_int8, kv_dequantise_int8, cross_attn_int8, cross_attn_int8_error_bound,
)
