"""MI355X-native prefill eviction pass of CAKE behind a C ABI (libcake.so).

The functions below are thin ctypes wrappers with the names of include/cake.h; all
arithmetic runs in the HIP kernels.  There is no CPU or PyTorch fallback: calling
anything without a built libcake.so raises.
"""
from .binding import (CAKE_BF16, CAKE_F32, CAKE_IND_MEAN, CAKE_IND_MEAN_PLUS_VAR, CAKE_IND_CUMULATIVE, CAKE_IND_MEAN_TIMES_VAR,  # noqa: F401
                      CAKE_IND_VAR, CakeError, cake_cascade_allocate, cake_compact_kv, cake_decode_step, cake_decode_step_workspace_bytes, cake_decode_update, cake_decode_update_static,  # noqa: F401
                      cake_evict_planned, cake_keep_counts, cake_layer_preference, cake_plan_bytes, cake_plan_eviction, cake_plan_layout, cake_profile_enable, cake_profile_read, cake_quantize_kv, cake_select_topk, cake_version, cake_window_scores,  # noqa: F401
                      cake_scores_chunk_keys, cake_window_scores_finish, cake_window_scores_lse, cake_window_scores_segment,  # noqa: F401
                      cake_workspace_bytes, make_params, make_shape, ptr_table)
from .driver import CacheQuantizer, CascadeSession, DecodeCache, DeviceCascade, DecodeSlots, EvictionPass, PassResult  # noqa: F401
