"""Decode-phase maintenance on the GPU against the oracle: cake_decode_update alone, and a few
generation steps through the driver (append, update, evict one row per head)."""
import numpy as np
import pytest
import torch

from oracle import cake_oracle as co
from synth import CONFIGS, make_config_inputs

from gpu_util import assert_close, host64, load_cake, oracle_params, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


@pytest.mark.parametrize("dtype,d,h_q,h_kv,window,B,pool", [(torch.bfloat16, 128, 8, 2, 32, 2, 7),
                                                            (torch.float32, 64, 4, 2, 32, 1, 1),
                                                            (torch.bfloat16, 64, 5, 1, 64, 1, 3),
                                                            (torch.float32, 128, 8, 1, 64, 2, 5)])
def test_decode_update_matches_oracle(cake, dtype, d, h_q, h_kv, window, B, pool):
    say(f"decode update {dtype} d={d} G={h_q // h_kv}")
    gen = torch.Generator().manual_seed(31)
    cur = [777, 300][:B]                                   # ragged batch: rows past a sequence's own count are unused
    cap = max(cur)
    rows = cap + window
    k = torch.randn(B, h_kv, rows, d, generator=gen).to(dtype).to(DEV)
    q = (torch.randn(B, h_q, d, generator=gen) * 3).to(dtype).to(DEV)
    ind0 = (torch.rand(B, h_kv, cap, generator=gen) * 2e-4).to(DEV)       # the size of one step's increments
    ind0[:, :, ::5] = 0.0                                                    # ... and rows that start from nothing
    ind = ind0.clone()
    params = cake.make_params(pool_kernel=pool)
    shape = cake.make_shape(B, 1, h_q, h_kv, d, rows, window, dtype)
    ws = torch.empty(cake.cake_workspace_bytes(shape), dtype=torch.uint8, device=DEV)
    cake.cake_decode_update(shape, params, cake.ptr_table([q]), [q.stride(0), q.stride(1)], cake.ptr_table([k]),
                            [[k.stride(0), k.stride(1), k.stride(2)]], cur, cake.ptr_table([ind]), ws)
    torch.cuda.synchronize()
    for b in range(B):
        n = cur[b] + window
        want = co.decode_update(host64(q[b]), host64(k[b, :, :n]), host64(ind0[b, :, : cur[b]]), window, oracle_params(params))
        assert_close(ind[b, :, : cur[b]].cpu().numpy(), want, f"updated indicator b={b}")
        assert torch.equal(ind[b, :, cur[b]:], ind0[b, :, cur[b]:])          # entries past cur_len untouched


def test_generation_steps_keep_every_layer_at_its_budget(cake):
    say("decode: generation steps after a prefill pass")
    cfg = CONFIGS[2].scaled(n_layers=3, seq_len=1200, total_budget=3 * 200)
    inp = make_config_inputs(cfg, device=DEV)
    L, S_w = cfg.n_layers, cfg.window
    q = [inp["q_win"][l] for l in range(L)]
    k = [inp["k"][l] for l in range(L)]
    v = [inp["v"][l] for l in range(L)]
    res = cake.EvictionPass(q, k, v, cfg.total_budget).run()
    torch.cuda.synchronize()
    cache = cake.DecodeCache(res, cfg.n_q_heads, S_w)
    oracle_cache = [{"k": host64(res.k_out[l][0]), "v": host64(res.v_out[l][0]),
                     "ind": host64(res.ind_out[l][0, :, : int(res.keep[l, 0])])} for l in range(L)]
    p = oracle_params(cache.params)
    gen = torch.Generator().manual_seed(77)
    for step in range(4):
        for l in range(L):
            qn = (torch.randn(1, cfg.n_q_heads, cfg.head_dim, generator=gen) * 2).to(torch.bfloat16).to(DEV)
            kn = torch.randn(1, cfg.n_kv_heads, cfg.head_dim, generator=gen).to(torch.bfloat16).to(DEV)
            vn = torch.randn(1, cfg.n_kv_heads, cfg.head_dim, generator=gen).to(torch.bfloat16).to(DEV)
            n_k = int(res.keep[l, 0])
            gpu_before = {"k": host64(cache.k[l][0]), "v": host64(cache.v[l][0]), "ind": host64(cache.ind[l][0])}
            cache.step(l, qn, kn, vn)
            torch.cuda.synchronize()
            assert cache.k[l].shape[2] == n_k + S_w and cache.ind[l].shape[2] == n_k       # size unchanged
            # the oracle's step from the GPU's state before the step: the same rows must go
            # unless the two lowest indicators are within the tolerance of each other
            want = co.decode_step(host64(qn[0]), gpu_before, host64(kn[0]), host64(vn[0]), S_w, p)
            got_idx = cache.last_idx[0, :, :n_k].cpu().numpy()
            for g in range(cfg.n_kv_heads):
                if not np.array_equal(got_idx[g], want["idx"][g]):
                    full = np.concatenate([gpu_before["ind"][g], [0.0]])
                    upd = co.decode_update(host64(qn[0]), np.concatenate([gpu_before["k"], host64(kn[0])[:, None]], axis=1),
                                           np.stack([np.concatenate([r, [0.0]]) for r in gpu_before["ind"]]), S_w, p)[g]
                    lost_gpu = np.setdiff1d(np.arange(n_k + 1), got_idx[g])
                    lost_ref = np.setdiff1d(np.arange(n_k + 1), want["idx"][g])
                    assert abs(upd[lost_gpu[0]] - upd[lost_ref[0]]) <= 2 * 1e-3 * abs(upd[lost_ref[0]]) + 1e-30, full.shape
                sel = got_idx[g]
                k_full = np.concatenate([gpu_before["k"][g], host64(kn[0])[g][None]], axis=0)
                np.testing.assert_array_equal(host64(cache.k[l][0, g]), co.compact(k_full, sel, S_w))
            assert_close(host64(cache.ind[l][0]), np.stack([want["ind"][g] if np.array_equal(got_idx[g], want["idx"][g])
                                                            else host64(cache.ind[l][0, g]) for g in range(cfg.n_kv_heads)]),
                         "indicator after the step")
            # the oracle's own trajectory (from its own state) agrees on the indicator values
            oracle_cache[l] = co.decode_step(host64(qn[0]), oracle_cache[l], host64(kn[0]), host64(vn[0]), S_w, p)
