"""MI355X-native SparK hot path: channel pruning of the key cache at prefill and decode
attention over the packed cache.  Thin ctypes binding over ``libspark_hip.so`` (C ABI in
``include/spark.h``); every step of the path runs in the library's HIP kernels."""
from .binding import (SparkDesc, decode_attn, decode_splits, decode_workspace_bytes, decode_workspace_init,
                      new_decode_workspace, lib_path,
                      load, packed_bytes, probe_read, decode_timeline, prune, unpack, SparkError,
                      packed_values_bytes, prune_values, unpack_values, decode_attn_values, decode_attn_tail, decode_attn_values_tail,
                      decode_attn_sampled, unpack_stats, check_packed, ERR_MISMATCH, packed_topp_bytes, prune_topp, decode_attn_topp, unpack_topp, decode_attn_static, STATIC_WORKSPACE_BYTES, RECOVER_GAUSSIAN, RECOVER_EXPONENTIAL,
                      PACK_BF16, PACK_INT8, OUT_BF16, OUT_F32)

__all__ = ["SparkDesc", "decode_attn", "decode_splits", "decode_workspace_bytes", "decode_workspace_init",
           "new_decode_workspace", "lib_path", "load",
           "packed_bytes", "probe_read", "decode_timeline", "prune", "unpack", "SparkError", "packed_values_bytes", "prune_values",
           "unpack_values", "decode_attn_values", "decode_attn_tail", "decode_attn_values_tail", "decode_attn_sampled", "unpack_stats", "check_packed", "ERR_MISMATCH", "packed_topp_bytes", "prune_topp", "decode_attn_topp", "unpack_topp", "decode_attn_static", "STATIC_WORKSPACE_BYTES", "RECOVER_GAUSSIAN",
           "RECOVER_EXPONENTIAL", "PACK_BF16", "PACK_INT8", "OUT_BF16",
           "OUT_F32"]
