"""Host-only checks of libcake: it loads, exports what include/cake.h declares, rejects bad
arguments before touching the GPU, and its allocator equals the oracle's exactly."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import cake_oracle as co

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def cake():
    import paper_2503_12491_amd as pkg
    from paper_2503_12491_amd import _ffi
    if not os.path.exists(_ffi.LIB_PATH):
        from paper_2503_12491_amd.build import build
        build()
    return pkg


def test_library_exports_every_declared_symbol(cake):
    from paper_2503_12491_amd import _ffi
    header = open(os.path.join(ROOT, "include", "cake.h")).read()
    declared = set(re.findall(r"\b(cake_[a-z_]+)\s*\(", header))
    assert {"cake_window_scores", "cake_window_scores_lse", "cake_layer_preference", "cake_cascade_allocate", "cake_select_topk",
            "cake_compact_kv", "cake_decode_update", "cake_decode_update_static", "cake_workspace_bytes", "cake_last_error", "cake_version",
            "cake_profile_enable", "cake_profile_read"} <= declared
    lib = ctypes.CDLL(_ffi.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert set(_ffi._SIGNATURES) == declared
    assert cake.cake_version() >= 100


def test_allocator_matches_oracle_exactly(cake):
    rng = np.random.default_rng(100)
    for trial in range(400):
        m1 = int(rng.integers(1, 65))
        window = int(rng.choice([1, 2, 32, 64]))
        n = int(rng.integers(window + 1, 3000))
        total = int(rng.integers(m1 * window, m1 * n + 100))
        kind = trial % 4
        if kind == 0:
            pref = rng.random(m1)
        elif kind == 1:
            pref = rng.choice([0.0, 0.5, 1.0, 1.0, 2.0, 3.0], size=m1).astype(float)   # ties, zeros
        elif kind == 2:
            pref = np.exp(rng.normal(0, 4, size=m1))                                    # wide spread
        else:
            pref = np.full(m1, float(rng.random()) + 0.1)                                # all equal
        want = co.cascade_allocate(pref, total, window, n)
        got = cake.cake_cascade_allocate(pref, total, window, n)
        assert got == want, (trial, list(pref), total, window, n)


def test_allocator_paper_scale(cake):
    rng = np.random.default_rng(101)
    pref = np.exp(rng.normal(0, 2, size=32))
    want = co.cascade_allocate(pref, 65536, 64, 131072)
    got = cake.cake_cascade_allocate(pref, 65536, 64, 131072)
    assert got == want and sum(got) == 65536
    # stage-wise (Eq. 9): budgets never grow as layers are admitted
    prev = None
    for m in range(32):
        cur = cake.cake_cascade_allocate(pref[: m + 1], 65536, 64, 131072)
        assert cur == co.cascade_allocate(pref[: m + 1], 65536, 64, 131072)
        if prev is not None:
            assert all(c <= p for c, p in zip(cur, prev))
        prev = cur


def test_allocator_errors(cake):
    E = cake.CakeError
    with pytest.raises(E):
        cake.cake_cascade_allocate([1.0, 1.0], 63, 32, 100)          # below the windows
    with pytest.raises(E):
        cake.cake_cascade_allocate([1.0, float("nan")], 640, 32, 100)
    with pytest.raises(E):
        cake.cake_cascade_allocate([1.0, -2.0], 640, 32, 100)
    with pytest.raises(E):
        cake.cake_cascade_allocate([1.0], 640, 32, 32)               # N <= S_w
    assert cake.cake_cascade_allocate([0.0, 0.0, 0.0], 300, 32, 5000) == [100, 100, 100]
    assert cake.cake_cascade_allocate([1.0, 3.0], 10_000, 32, 100) == [100, 100]


def test_shape_and_argument_errors_are_reported_on_the_host(cake):
    E = cake.CakeError
    ok = cake.make_shape(1, 2, 4, 2, 64, 1024, 32, cake.CAKE_F32)
    assert cake.cake_workspace_bytes(ok) > 0
    for bad in (cake.make_shape(1, 2, 4, 2, 64, 32, 32, cake.CAKE_F32),      # N <= S_w
                cake.make_shape(1, 2, 4, 2, 96, 1024, 32, cake.CAKE_F32),     # head_dim
                cake.make_shape(1, 2, 4, 2, 64, 1024, 48, cake.CAKE_F32),     # window
                cake.make_shape(1, 2, 5, 2, 64, 1024, 32, cake.CAKE_F32),     # H_q % H_kv
                cake.make_shape(1, 2, 18, 2, 64, 1024, 32, cake.CAKE_F32),    # group > 8
                cake.make_shape(1, 2, 4, 2, 64, 1024, 32, 7),                 # dtype
                cake.make_shape(0, 2, 4, 2, 64, 1024, 32, cake.CAKE_F32)):
        with pytest.raises(E) as info:
            cake.cake_workspace_bytes(bad)
        assert info.value.code in (-1, -2) and str(info.value)
    # NULL tables / workspace are refused before any launch
    from paper_2503_12491_amd import binding as C
    params = cake.make_params()
    rc = C.load().cake_window_scores(ctypes.byref(ok), ctypes.byref(params), None, None, None, None, None, None, 0, None)
    assert rc == -1 and b"NULL" in C.load().cake_last_error()
    rc = C.load().cake_select_topk(ctypes.byref(ok), None, None, None, None, None, 0, None)
    assert rc == -1
    rc = C.load().cake_compact_kv(ctypes.byref(ok), None, None, None, None, None, None, None, None, None, None, None)
    assert rc == -1
    rc = C.load().cake_layer_preference(ctypes.byref(ok), ctypes.byref(params), None, 0, None, None, None)
    assert rc == -1
    rc = C.load().cake_window_scores_lse(ctypes.byref(ok), ctypes.byref(params), None, None, None, None, None, None, None, 0, None)
    assert rc == -1 and b"row_lse" in C.load().cake_last_error()
    rc = C.load().cake_decode_update(ctypes.byref(ok), ctypes.byref(params), None, None, None, None, None, None, None, 0, None)
    assert rc == -1 and b"NULL" in C.load().cake_last_error()
    # parameter checks: indicator mode, pooling width, decode lengths beyond the cache capacity
    one = (ctypes.c_int64 * 3)(64, 64, 64)
    tbl = ctypes.c_void_p(256)                      # never dereferenced: the call fails before any launch
    bad_mode = cake.make_params(indicator_mode=9)
    rc = C.load().cake_window_scores(ctypes.byref(ok), ctypes.byref(bad_mode), tbl, tbl, one, one, tbl, tbl, 1 << 30, None)
    assert rc == -1 and b"indicator_mode" in C.load().cake_last_error()
    bad_pool = cake.make_params(pool_kernel=4)
    rc = C.load().cake_window_scores(ctypes.byref(ok), ctypes.byref(bad_pool), tbl, tbl, one, one, tbl, tbl, 1 << 30, None)
    assert rc == -1 and b"pool_kernel" in C.load().cake_last_error()
    too_long = (ctypes.c_int32 * 2)(1024, 10)        # cur_len > seq_len - window
    two = (ctypes.c_int64 * 2)(256, 64)
    six = (ctypes.c_int64 * 6)(64, 64, 64, 64, 64, 64)
    rc = C.load().cake_decode_update(ctypes.byref(ok), ctypes.byref(params), tbl, two, tbl, six, too_long, tbl, tbl, 1 << 30, None)
    assert rc == -1 and b"cur_len" in C.load().cake_last_error()
    rc = C.load().cake_window_scores(ctypes.byref(ok), ctypes.byref(params), tbl, tbl, one, one, tbl, tbl, 16, None)
    assert rc == -3                                   # workspace too small


def test_workspace_grows_with_the_problem(cake):
    small = cake.cake_workspace_bytes(cake.make_shape(1, 2, 4, 2, 64, 1024, 32, cake.CAKE_F32))
    big = cake.cake_workspace_bytes(cake.make_shape(1, 32, 32, 8, 128, 131072, 64, cake.CAKE_BF16))
    assert small < big
    n_p = 131072 - 64
    assert big >= 32 * 8 * n_p * 4          # at least the un-pooled indicator
    assert big < 400 * 2 ** 20


def test_keep_counts_clamp_budget_minus_window(cake):
    """cake_keep_counts: k = clamp(B_l - S_w, 0, cur_len), the count the oracle's evict() retains."""
    from paper_2503_12491_amd import binding as C
    budgets = np.array([[64, 100], [3000, 10], [65, 700]])
    cur = np.array([[500, 20], [500, 0], [1, 636]])
    got = C.cake_keep_counts(budgets, cur, 64)
    assert got.tolist() == [[0, 20], [500, 0], [1, 636]]
    assert C.cake_keep_counts(budgets, 1000, 64).tolist() == [[0, 36], [1000, 0], [1, 636]]
    # the oracle keeps budget - window prefix rows when the budget includes the window
    k = np.arange(40 * 3, dtype=np.float64).reshape(40, 3)
    ind = np.linspace(1.0, 0.0, 32)
    k_hat, _, _, idx = co.evict(k, k, ind, 8 + 5, 8)
    assert k_hat.shape[0] == 13 and int(C.cake_keep_counts(np.array([13]), 32, 8)[0]) == idx.shape[0]
    with pytest.raises(C.CakeError):
        C.cake_keep_counts(np.array([5]), np.array([-1]), 4)


def test_segment_calls_reject_bad_arguments_on_the_host(cake):
    """cake_window_scores_segment / _finish validate before anything is launched: pass number,
    segment alignment to the chunk of cake_scores_chunk_keys, range, NULL tables, workspace."""
    from paper_2503_12491_amd import binding as C
    import torch
    shape = C.make_shape(1, 2, 4, 2, 64, 1024 + 77, 32, torch.float32)
    params = C.make_params()
    chunk = C.cake_scores_chunk_keys(shape)
    assert chunk == 256
    assert C.cake_scores_chunk_keys(C.make_shape(1, 1, 32, 8, 128, 131072, 64, torch.bfloat16)) == 2048
    lib = C.load()
    one = (ctypes.c_int64 * 3)(4096, 1024, 64)
    tbl = ctypes.c_void_p(256)            # never dereferenced: every call below fails validation first
    ws = ctypes.c_void_p(1 << 20)

    def seg(which, lo, cnt, q=tbl, k=tbl, wsp=ws, nbytes=1 << 30):
        return lib.cake_window_scores_segment(ctypes.byref(shape), ctypes.byref(params), which, lo, cnt, q, k, one, one,
                                              wsp, nbytes, None)
    assert seg(3, 0, chunk) == -1 and b"pass" in lib.cake_last_error()
    assert seg(1, chunk // 2, chunk) == -1 and b"multiple of the chunk" in lib.cake_last_error()
    assert seg(1, 0, chunk + 1) == -1
    assert seg(2, 0, 0) == -1
    assert seg(1, chunk, 1024 + 77) == -1                 # runs past seq_len
    assert seg(1, 0, chunk, q=None) == -1
    assert seg(1, 0, chunk, nbytes=16) == -3
    assert seg(1, 0, chunk, wsp=None) == -3
    fin = lib.cake_window_scores_finish
    assert fin(ctypes.byref(shape), ctypes.byref(params), 0, tbl, ws, 1 << 30, None) == -1
    assert fin(ctypes.byref(shape), ctypes.byref(params), 2, None, ws, 1 << 30, None) == -1
    assert fin(ctypes.byref(shape), ctypes.byref(params), 1, None, ws, 16, None) == -3
