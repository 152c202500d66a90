"""CPU oracle for the decode-attention step (TEST INFRASTRUCTURE ONLY).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares nothing with the GPU library: its arithmetic lives in
oracle/sw_oracle.c (plain C, fp64), built here with gcc and called via ctypes.
"""
from .binding import (build, decode_attn, decode_attn_paged, kv_append, kv_append_paged,
                      prefill_attn, mixed_attn, mixed_attn_paged, kv_store, kv_pack, kv_span_plan,
                      half_to_double, max_threads, lib_path)

__all__ = ["build", "decode_attn", "decode_attn_paged", "kv_append", "kv_append_paged", "prefill_attn", "mixed_attn", "mixed_attn_paged", "kv_store", "kv_pack", "kv_span_plan",
           "half_to_double", "max_threads", "lib_path"]
