"""cake_decode_update_static (the entry point that takes no workspace and allocates nothing)
against cake_decode_update on the same inputs, through the C ABI: two calls in a row, the
second on a smaller problem, both compared bit for bit (the two entry points run the same
kernels and differ only in where the chunks' partial sums are kept)."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_util import load_cake, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _problem(seed, L, B, H_q, H_kv, d, cur_max, S_w):
    gen = torch.Generator().manual_seed(seed)
    rng = np.random.default_rng(seed)
    rows = cur_max + S_w
    k = [torch.randn(B, H_kv, rows, d, generator=gen).to(torch.bfloat16).to(DEV) for _ in range(L)]
    q = [(torch.randn(B, H_q, d, generator=gen) * 2).to(torch.bfloat16).to(DEV) for _ in range(L)]
    ind = [torch.rand(B, H_kv, cur_max, generator=gen).to(DEV) for _ in range(L)]
    cur = rng.integers(max(cur_max // 2, 1), cur_max + 1, size=(L, B))
    cur[:, 0] = cur_max                      # the row capacity of `ind` is max_b cur_len
    return q, k, ind, [int(c) for c in cur.reshape(-1)]


def _run_both(cake, seed, L, B, H_q, H_kv, d, cur_max, S_w):
    from paper_2503_12491_amd import binding as C
    q, k, ind, cur = _problem(seed, L, B, H_q, H_kv, d, cur_max, S_w)
    shape = C.make_shape(B, L, H_q, H_kv, d, cur_max + S_w, S_w, torch.bfloat16)
    params = C.make_params()
    tq, tk = C.ptr_table(q), C.ptr_table(k)
    qs = [q[0].stride(0), q[0].stride(1)]
    ks = [[t.stride(0), t.stride(1), t.stride(2)] for t in k]
    ind_a = [t.clone() for t in ind]
    ind_b = [t.clone() for t in ind]
    ws = torch.empty(C.cake_workspace_bytes(shape), dtype=torch.uint8, device=DEV)
    C.cake_decode_update(shape, params, tq, qs, tk, ks, cur, C.ptr_table(ind_a), ws)
    C.cake_decode_update_static(shape, params, tq, qs, tk, ks, cur, C.ptr_table(ind_b))
    torch.cuda.synchronize()
    for l in range(L):
        assert torch.equal(ind_a[l], ind_b[l]), f"layer {l}"
        assert not torch.equal(ind_a[l], ind[l])          # the update did something


def test_static_scratch_entry_point_matches_workspace_entry_point():
    cake = load_cake()
    say("no-alloc decode update: 4 layers x 2 sequences x 8 heads, caches of up to 3000 rows")
    _run_both(cake, 1, L=4, B=2, H_q=32, H_kv=8, d=128, cur_max=3000, S_w=32)
    say("no-alloc decode update: second call, smaller (1 layer, 300 rows), same scratch")
    _run_both(cake, 2, L=1, B=1, H_q=8, H_kv=2, d=64, cur_max=300, S_w=32)


def test_static_scratch_entry_point_rejects_oversized_shapes():
    load_cake()
    from paper_2503_12491_amd import binding as C
    # 64 layers x 4 x 8 heads x ceil(32768/256) chunks = 262144 entries: beyond the built-in scratch
    shape = C.make_shape(4, 64, 40, 8, 128, 32768, 32, torch.bfloat16)
    params = C.make_params()
    one = torch.zeros(64, dtype=torch.int64, device=DEV)
    with pytest.raises(C.CakeError) as err:
        C.cake_decode_update_static(shape, params, one, [128, 128], one, [[128, 128, 128]] * 64, [0] * 256, one)
    assert err.value.code == -2 and "built-in scratch" in str(err.value)
