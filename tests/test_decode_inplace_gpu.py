"""In-place decode step (cake_decode_step) against the oracle's decode_step, through the slot list:
after every step the cache read in logical order must be the oracle's cache computed from the
logical cache before the step: the same row evicted (unless two candidates lie within the
tolerance of each other), K and V bit-exact, indicators within 1e-3."""
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


def _check_steps(cake, cfg, n_steps, seed):
    inp = make_config_inputs(cfg, device=DEV)
    L, S_w, B = cfg.n_layers, cfg.window, cfg.batch
    res = cake.EvictionPass([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)],
                            [inp["v"][l] for l in range(L)], cfg.total_budget).run()
    torch.cuda.synchronize()
    slots = cake.DecodeSlots(res, cfg.n_q_heads, S_w)
    p = oracle_params(slots.params)
    gen = torch.Generator().manual_seed(seed)
    slot_addr = [(t.data_ptr(), u.data_ptr()) for t, u in zip(slots.k, slots.v)]
    for step in range(n_steps):
        for l in range(L):
            qn = (torch.randn(B, cfg.n_q_heads, cfg.head_dim, generator=gen) * 2).to(cfg.torch_dtype).to(DEV)
            kn = torch.randn(B, cfg.n_kv_heads, cfg.head_dim, generator=gen).to(cfg.torch_dtype).to(DEV)
            vn = torch.randn(B, cfg.n_kv_heads, cfg.head_dim, generator=gen).to(cfg.torch_dtype).to(DEV)
            before = [slots.logical(l, b) for b in range(B)]
            before = [(host64(k_), host64(v_), host64(i_)) for k_, v_, i_, _ in before]
            slots.step(l, qn, kn, vn)
            torch.cuda.synchronize()
            for b in range(B):
                k0, v0, i0 = before[b]
                cur = i0.shape[1]
                assert cur == int(res.keep[l, b])                                     # the size never changes
                want = co.decode_step(host64(qn[b]), {"k": k0, "v": v0, "ind": i0}, host64(kn[b]), host64(vn[b]), S_w, p)
                k1, v1, i1, evicted = slots.logical(l, b)
                k1, v1, i1 = host64(k1), host64(v1), host64(i1)
                upd = co.decode_update(host64(qn[b]), np.concatenate([k0, host64(kn[b])[:, None]], axis=1),
                                       np.concatenate([i0, np.zeros((cfg.n_kv_heads, 1))], axis=1), S_w, p)
                for g in range(cfg.n_kv_heads):
                    lost_ref = np.setdiff1d(np.arange(cur + 1), want["idx"][g])[0]
                    e = int(evicted[g])
                    if e != lost_ref:      # two candidates within the tolerance of each other may change places
                        assert abs(upd[g, e] - upd[g, lost_ref]) <= 2 * 1e-3 * abs(upd[g, lost_ref]) + 1e-30, (l, b, g, e, lost_ref)
                    sel = np.delete(np.arange(cur + 1), e)
                    k_full = np.concatenate([k0[g], host64(kn[b])[g][None]], axis=0)
                    v_full = np.concatenate([v0[g], host64(vn[b])[g][None]], axis=0)
                    np.testing.assert_array_equal(k1[g], co.compact(k_full, sel, S_w))
                    np.testing.assert_array_equal(v1[g], co.compact(v_full, sel, S_w))
                    assert_close(i1[g], upd[g][sel], f"indicator after the step l={l} b={b} g={g}")
    # nothing was reallocated: the slots are where they were
    assert slot_addr == [(t.data_ptr(), u.data_ptr()) for t, u in zip(slots.k, slots.v)]


def test_in_place_steps_match_the_oracle_llama_shape(cake):
    say("in-place decode: 3 layers, 5 steps, G = 4, bf16")
    _check_steps(cake, CONFIGS[2].scaled(n_layers=3, seq_len=1200, total_budget=3 * 300), n_steps=5, seed=5)


def test_in_place_steps_match_the_oracle_ragged_batch(cake):
    say("in-place decode: batch of 3 with per-sequence budgets, G = 5")
    _check_steps(cake, CONFIGS[5].scaled(n_layers=2, batch=3, seq_len=700, total_budget=2 * 150), n_steps=3, seed=6)


def test_in_place_steps_match_the_oracle_fp32_tiny(cake):
    say("in-place decode: tiny fp32 config")
    _check_steps(cake, CONFIGS[1], n_steps=4, seed=7)


def test_all_layers_in_one_call_equal_layer_by_layer(cake):
    """DecodeSlots.step_all (one cake_decode_step call for all layers, per-layer slot strides and
    capacities) leaves every buffer exactly as the layer-by-layer steps do."""
    say("in-place decode: all layers in one call vs layer by layer")
    cfg = CONFIGS[2].scaled(n_layers=5, seq_len=1500, total_budget=5 * 260)
    inp = make_config_inputs(cfg, device=DEV)
    L, B = cfg.n_layers, cfg.batch
    res = cake.EvictionPass([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)],
                            [inp["v"][l] for l in range(L)], cfg.total_budget).run()
    torch.cuda.synchronize()
    assert len(set(int(x) for x in res.keep[:, 0])) > 1                  # layers of different capacities
    one, many = cake.DecodeSlots(res, cfg.n_q_heads, cfg.window), cake.DecodeSlots(res, cfg.n_q_heads, cfg.window)
    gen = torch.Generator().manual_seed(3)
    for step in range(4):
        qn = (torch.randn(L, B, cfg.n_q_heads, cfg.head_dim, generator=gen) * 2).to(cfg.torch_dtype).to(DEV)
        kn = torch.randn(L, B, cfg.n_kv_heads, cfg.head_dim, generator=gen).to(cfg.torch_dtype).to(DEV)
        vn = torch.randn(L, B, cfg.n_kv_heads, cfg.head_dim, generator=gen).to(cfg.torch_dtype).to(DEV)
        for l in range(L):
            one.step(l, qn[l], kn[l], vn[l])
        many.step_all(qn, kn, vn)
        torch.cuda.synchronize()
        for l in range(L):
            for name in ("k", "v", "ind", "order", "state"):
                assert torch.equal(getattr(one, name)[l], getattr(many, name)[l]), (step, l, name)
