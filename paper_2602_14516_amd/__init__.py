"""MI355X-native batched incremental-prefill attention over a paged KV cache.

The package is a thin binding over libampd.so (hand-written HIP for gfx950 behind a C ABI,
see include/ampd.h).  There is no CPU or PyTorch fallback: if the shared library has not
been built, importing the binding raises.
"""
from .binding import (KVCache, kv_append, kv_pack, kv_unpack, incr_prefill_attn, mixed_batch_attn, paged_attn,
                      init, mixed_batch_attn_static, static_workspace_limit, workspace_bytes, plan_describe, plan_items, set_timing, last_timing,
                      status_string, version, AmpdError, lib, LIB_PATH, EXPORTED_SYMBOLS)

__all__ = ["KVCache", "kv_append", "kv_pack", "kv_unpack", "incr_prefill_attn", "mixed_batch_attn", "paged_attn",
           "init", "mixed_batch_attn_static", "static_workspace_limit", "workspace_bytes", "plan_describe", "plan_items", "set_timing", "last_timing",
           "status_string", "version", "AmpdError", "lib", "LIB_PATH", "EXPORTED_SYMBOLS"]
