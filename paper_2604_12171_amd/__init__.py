"""MI355X-native hot path of PipeLive: paged-attention decode over a
resizable block-list KV cache, in-place KV resize/compaction and incremental
KV patching, as hand-written HIP kernels behind a C ABI (include/pipelive.h).
This package is the thin Python binding of that library."""
from .binding import *  # noqa: F401,F403
from .binding import (KVRegion, Arena, PipeliveError, load, pipelive_kv_append, pipelive_kv_clear_status,  # noqa: F401
                      pipelive_kv_mark_dirty, pipelive_kv_patch_apply, pipelive_kv_patch_collect,
                      pipelive_kv_read_state, pipelive_kv_resize, pipelive_max_blocks,
                      pipelive_paged_attn_decode, pipelive_paged_attn_prefill, pipelive_patch_max_blocks, pipelive_plan_reconfig,
                      pipelive_converged)
