"""Python names for the C ABI of libcake (include/cake.h).  Argument marshalling only."""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence

import torch

from ._ffi import cake_params, cake_shape, load

CAKE_BF16, CAKE_F32 = 0, 1


class CakeError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libcake error {code}: {message}")
        self.code = code


def _check(rc: int) -> None:
    if rc != 0:
        raise CakeError(rc, load().cake_last_error().decode())


def make_shape(batch, n_layers, n_q_heads, n_kv_heads, head_dim, seq_len, window, dtype) -> cake_shape:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.bfloat16: CAKE_BF16, torch.float32: CAKE_F32}[dtype]
    return cake_shape(batch, n_layers, n_q_heads, n_kv_heads, head_dim, seq_len, window, dtype)


CAKE_IND_MEAN_PLUS_VAR, CAKE_IND_MEAN, CAKE_IND_VAR, CAKE_IND_MEAN_TIMES_VAR, CAKE_IND_CUMULATIVE = 0, 1, 2, 3, 4


def make_params(scale=0.0, gamma=200.0, tau1=1.0, tau2=1.0, var_correction=1, pool_kernel=7,
                indicator_mode=CAKE_IND_MEAN_PLUS_VAR) -> cake_params:
    return cake_params(scale, gamma, tau1, tau2, var_correction, pool_kernel, indicator_mode)


def ptr_table(tensors: Sequence[torch.Tensor]) -> torch.Tensor:
    """Device array of the tensors' base addresses (one per layer)."""
    dev = tensors[0].device
    return torch.tensor([t.data_ptr() for t in tensors], dtype=torch.int64).to(dev)


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        return x.data_ptr()
    return int(x)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _i64(vals):
    return (ctypes.c_int64 * len(vals))(*[int(v) for v in vals])


def _i32(vals):
    return (ctypes.c_int32 * len(vals))(*[int(v) for v in vals])


def cake_version() -> int:
    return load().cake_version()


def cake_workspace_bytes(shape: cake_shape) -> int:
    out = ctypes.c_size_t(0)
    _check(load().cake_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def cake_window_scores(shape, params, q_win, k, q_strides, k_strides, indicator, workspace, stream=None) -> None:
    _check(load().cake_window_scores(ctypes.byref(shape), ctypes.byref(params), _ptr(q_win), _ptr(k),
                                     _i64(q_strides), _i64(k_strides), _ptr(indicator), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)))


def cake_window_scores_lse(shape, params, q_win, k, q_strides, k_strides, row_lse, indicator, workspace,
                           stream=None) -> None:
    _check(load().cake_window_scores_lse(ctypes.byref(shape), ctypes.byref(params), _ptr(q_win), _ptr(k),
                                         _i64(q_strides), _i64(k_strides), _ptr(row_lse), _ptr(indicator),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(),
                                         _stream(stream)))


def cake_scores_chunk_keys(shape: cake_shape) -> int:
    out = ctypes.c_int32(0)
    _check(load().cake_scores_chunk_keys(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def cake_window_scores_segment(shape, params, which_pass, key_begin, key_count, q_win, k_segment, q_strides, k_strides,
                               workspace, stream=None) -> None:
    _check(load().cake_window_scores_segment(ctypes.byref(shape), ctypes.byref(params), which_pass, key_begin, key_count,
                                             _ptr(q_win), _ptr(k_segment), _i64(q_strides), _i64(k_strides),
                                             _ptr(workspace), workspace.numel() * workspace.element_size(),
                                             _stream(stream)))


def cake_window_scores_finish(shape, params, which_pass, indicator, workspace, stream=None) -> None:
    _check(load().cake_window_scores_finish(ctypes.byref(shape), ctypes.byref(params), which_pass, _ptr(indicator),
                                            _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream)))


def cake_layer_preference(shape, params, workspace, pref, hv=None, stream=None) -> None:
    _check(load().cake_layer_preference(ctypes.byref(shape), ctypes.byref(params), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _ptr(pref), _ptr(hv),
                                        _stream(stream)))


def cake_keep_counts(budgets, cur_len, window: int):
    """Prefix tokens kept per entry; budgets and cur_len are integer arrays of one shape (returned shape too)."""
    import numpy as np
    b = np.ascontiguousarray(budgets, dtype=np.int32)
    c = np.ascontiguousarray(np.broadcast_to(cur_len, b.shape), dtype=np.int32)
    out = np.empty_like(b)
    as_p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    _check(load().cake_keep_counts(as_p(b), as_p(c), b.size, window, as_p(out)))
    return out.astype(np.int64)


def cake_cascade_allocate(pref: Sequence[float], total_budget: int, window: int, seq_len: int) -> list:
    n = len(pref)
    p = (ctypes.c_double * n)(*[float(x) for x in pref])
    out = (ctypes.c_int32 * n)()
    _check(load().cake_cascade_allocate(p, n, int(total_budget), int(window), int(seq_len), out))
    return list(out)


def cake_select_topk(shape, indicator, cur_len, k, idx, workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().cake_select_topk(ctypes.byref(shape), _ptr(indicator), _i32(cur_len), _i32(k), _ptr(idx),
                                   _ptr(workspace), ws_bytes, _stream(stream)))


def cake_plan_bytes(shape: cake_shape) -> int:
    out = ctypes.c_size_t(0)
    _check(load().cake_plan_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def cake_plan_eviction(shape, pref, total_budget, cur_len, pool_idx, pool_k, pool_v, pool_ind, plan, status,
                       stream=None) -> None:
    _check(load().cake_plan_eviction(ctypes.byref(shape), _ptr(pref), int(total_budget), _ptr(cur_len), _ptr(pool_idx),
                                     _ptr(pool_k), _ptr(pool_v), _ptr(pool_ind), _ptr(plan),
                                     plan.numel() * plan.element_size(), _ptr(status), _stream(stream)))


def cake_evict_planned(shape, indicator, k_in, v_in, kv_strides, plan, stream=None, compacted=None) -> None:
    """compacted: per layer 1 if its k_in/v_in are outputs of an earlier planned compaction (strides from the plan)."""
    flags = None if compacted is None else (ctypes.c_uint8 * len(compacted))(*[int(x) for x in compacted])
    _check(load().cake_evict_planned(ctypes.byref(shape), _ptr(indicator), _ptr(k_in), _ptr(v_in), _i64(kv_strides), flags,
                                     _ptr(plan), plan.numel() * plan.element_size(), _stream(stream)))


PLAN_PARTS = ("budgets", "keep", "cur_len", "cap_keep", "cap_cur", "copy_blocks", "idx", "k_out", "v_out", "ind_out")


def cake_plan_layout(shape: cake_shape) -> dict:
    """Byte offsets of the plan's parts for (shape.n_layers, shape.batch), by name."""
    out = (ctypes.c_size_t * 10)()
    _check(load().cake_plan_layout(ctypes.byref(shape), out))
    return dict(zip(PLAN_PARTS, [int(x) for x in out]))


def plan_fields(plan_host, n_layers: int, batch: int):
    """budgets, keep, cur_len [L, B] and cap_keep [L] of a plan copied to the host (a uint8 tensor)."""
    import numpy as np
    raw = plan_host.numpy().view(np.int32)
    lb = n_layers * batch
    budgets = raw[0:lb].reshape(n_layers, batch)
    keep = raw[lb:2 * lb].reshape(n_layers, batch)
    cur = raw[2 * lb:3 * lb].reshape(n_layers, batch)
    cap_keep = raw[3 * lb:3 * lb + n_layers]
    return budgets.astype(np.int64), keep.astype(np.int64), cur.astype(np.int64), cap_keep.astype(np.int64)


def cake_decode_update(shape, params, q_new, q_strides, k_cache, k_strides, cur_len, indicator, workspace,
                       stream=None) -> None:
    flat = [s for layer in k_strides for s in layer]
    _check(load().cake_decode_update(ctypes.byref(shape), ctypes.byref(params), _ptr(q_new), _i64(q_strides),
                                     _ptr(k_cache), _i64(flat), _i32(cur_len), _ptr(indicator), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)))


def cake_decode_step_workspace_bytes(shape: cake_shape) -> int:
    out = ctypes.c_size_t(0)
    _check(load().cake_decode_step_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def cake_decode_step(shape, params, q_new, q_strides, k_new, v_new, kv_new_strides, k_slots, v_slots, slot_strides,
                     indicator, order, state, cap, workspace, stream=None) -> None:
    """slot_strides: one [batch, head, slot] triple per layer of the call."""
    flat = [s for layer in slot_strides for s in layer]
    _check(load().cake_decode_step(ctypes.byref(shape), ctypes.byref(params), _ptr(q_new), _i64(q_strides), _ptr(k_new),
                                   _ptr(v_new), _i64(kv_new_strides), _ptr(k_slots), _ptr(v_slots), _i64(flat),
                                   _ptr(indicator), _ptr(order), _ptr(state), _i32(cap), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)))


def cake_decode_update_static(shape, params, q_new, q_strides, k_cache, k_strides, cur_len, indicator, stream=None) -> None:
    flat = [s for layer in k_strides for s in layer]
    _check(load().cake_decode_update_static(ctypes.byref(shape), ctypes.byref(params), _ptr(q_new), _i64(q_strides),
                                            _ptr(k_cache), _i64(flat), _i32(cur_len), _ptr(indicator), _stream(stream)))


def cake_compact_kv(shape, k_in, v_in, kv_strides, cur_len, k, idx, ind_in, k_out, v_out, ind_out,
                    stream=None) -> None:
    flat = [s for layer in kv_strides for s in layer]
    _check(load().cake_compact_kv(ctypes.byref(shape), _ptr(k_in), _ptr(v_in), _i64(flat), _i32(cur_len), _i32(k),
                                  _ptr(idx), _ptr(ind_in), _ptr(k_out), _ptr(v_out), _ptr(ind_out),
                                  _stream(stream)))


def cake_quantize_kv(shape, bits, k_hat, v_hat, kv_strides, keep, k_codes, k_scale, k_zero, v_codes, v_scale, v_zero,
                     stream=None) -> None:
    flat = [s for layer in kv_strides for s in layer]
    _check(load().cake_quantize_kv(ctypes.byref(shape), bits, _ptr(k_hat), _ptr(v_hat), _i64(flat), _i32(keep),
                                   _ptr(k_codes), _ptr(k_scale), _ptr(k_zero), _ptr(v_codes), _ptr(v_scale), _ptr(v_zero),
                                   _stream(stream)))


def cake_profile_enable(enable: bool) -> None:
    _check(load().cake_profile_enable(1 if enable else 0))


def cake_profile_read() -> list:
    """Milliseconds per cake_window_scores call, averaged over the calls since profiling was enabled:
    [pass 1, combine, pass 2, pooling] (with handed-over normalisers: [their import, 0, pass 2, pooling])."""
    out = (ctypes.c_float * 4)()
    _check(load().cake_profile_read(out))
    return list(out)
