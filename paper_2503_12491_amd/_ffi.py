"""ctypes loader for libcake.so.  Fails loudly when the library has not been built."""
from __future__ import annotations

import ctypes
import os

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcake.so")


class cake_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("batch", "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "seq_len", "window", "dtype")]


class cake_params(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_float), ("gamma", ctypes.c_float), ("tau1", ctypes.c_float),
                ("tau2", ctypes.c_float), ("var_correction", ctypes.c_int32), ("pool_kernel", ctypes.c_int32),
                ("indicator_mode", ctypes.c_int32)]


_P = ctypes.c_void_p
_SIGNATURES = {
    "cake_version": (ctypes.c_int, []),
    "cake_last_error": (ctypes.c_char_p, []),
    "cake_workspace_bytes": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(ctypes.c_size_t)]),
    "cake_window_scores": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), _P, _P,
                                          ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64), _P,
                                          _P, ctypes.c_size_t, _P]),
    "cake_window_scores_lse": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), _P, _P,
                                              ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64), _P, _P,
                                              _P, ctypes.c_size_t, _P]),
    "cake_scores_chunk_keys": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(ctypes.c_int32)]),
    "cake_window_scores_segment": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), ctypes.c_int32,
                                                  ctypes.c_int32, ctypes.c_int32, _P, _P,
                                                  ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
                                                  _P, ctypes.c_size_t, _P]),
    "cake_window_scores_finish": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), ctypes.c_int32,
                                                 _P, _P, ctypes.c_size_t, _P]),
    "cake_layer_preference": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), _P,
                                             ctypes.c_size_t, _P, _P, _P]),
    "cake_keep_counts": (ctypes.c_int, [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                        ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]),
    "cake_quantize_kv": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.c_int32, _P, _P, ctypes.POINTER(ctypes.c_int64),
                                        ctypes.POINTER(ctypes.c_int32), _P, _P, _P, _P, _P, _P, _P]),
    "cake_cascade_allocate": (ctypes.c_int, [ctypes.POINTER(ctypes.c_double), ctypes.c_int32, ctypes.c_int64,
                                             ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]),
    "cake_select_topk": (ctypes.c_int, [ctypes.POINTER(cake_shape), _P, ctypes.POINTER(ctypes.c_int32),
                                        ctypes.POINTER(ctypes.c_int32), _P, _P, ctypes.c_size_t, _P]),
    "cake_compact_kv": (ctypes.c_int, [ctypes.POINTER(cake_shape), _P, _P, ctypes.POINTER(ctypes.c_int64),
                                       ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), _P, _P,
                                       _P, _P, _P, _P]),
    "cake_plan_bytes": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(ctypes.c_size_t)]),
    "cake_plan_eviction": (ctypes.c_int, [ctypes.POINTER(cake_shape), _P, ctypes.c_int64, _P, _P, _P, _P, _P, _P,
                                          ctypes.c_size_t, _P, _P]),
    "cake_evict_planned": (ctypes.c_int, [ctypes.POINTER(cake_shape), _P, _P, _P, ctypes.POINTER(ctypes.c_int64),
                                          ctypes.POINTER(ctypes.c_uint8), _P, ctypes.c_size_t, _P]),
    "cake_plan_layout": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(ctypes.c_size_t)]),
    "cake_decode_update": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), _P,
                                          ctypes.POINTER(ctypes.c_int64), _P, ctypes.POINTER(ctypes.c_int64),
                                          ctypes.POINTER(ctypes.c_int32), _P, _P, ctypes.c_size_t, _P]),
    "cake_decode_step_workspace_bytes": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(ctypes.c_size_t)]),
    "cake_decode_step": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), _P,
                                        ctypes.POINTER(ctypes.c_int64), _P, _P, ctypes.POINTER(ctypes.c_int64), _P, _P,
                                        ctypes.POINTER(ctypes.c_int64), _P, _P, _P, ctypes.POINTER(ctypes.c_int32), _P,
                                        ctypes.c_size_t, _P]),
    "cake_decode_update_static": (ctypes.c_int, [ctypes.POINTER(cake_shape), ctypes.POINTER(cake_params), _P,
                                                 ctypes.POINTER(ctypes.c_int64), _P, ctypes.POINTER(ctypes.c_int64),
                                                 ctypes.POINTER(ctypes.c_int32), _P, _P]),
    "cake_profile_enable": (ctypes.c_int, [ctypes.c_int]),
    "cake_profile_read": (ctypes.c_int, [ctypes.POINTER(ctypes.c_float)]),
}

_lib = None


def load() -> ctypes.CDLL:
    """The loaded library.  Raises if libcake.so is absent: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_12491_amd.build` "
                "(hipcc, gfx950).  This package has no CPU or PyTorch fallback.")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib
