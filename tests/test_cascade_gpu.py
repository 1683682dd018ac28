"""Alg. 1 on the GPU: the cascading pass must end with the caches of the one-shot pass (Thm. 2),
stage budgets must never grow (Prop. 1) and must equal the oracle allocator fed the GPU's
preferences; the oracle's own Alg. 1 fed the GPU's indicators must retain the same positions."""
import numpy as np
import pytest
import torch

from oracle import cake_oracle as co
from synth import CONFIGS, make_config_inputs

from gpu_util import load_cake, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


def _run_both(cake, cfg):
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    args = ([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)], [inp["v"][l] for l in range(L)])
    shot = cake.EvictionPass(*args, cfg.total_budget).run()
    torch.cuda.synchronize()
    shot_k = [t.clone() for t in shot.k_out]
    shot_v = [t.clone() for t in shot.v_out]
    shot_i = [t.clone() for t in shot.ind_out]
    shot_idx = [t.clone() for t in shot.idx]
    casc = cake.EvictionPass(*args, cfg.total_budget).run_cascade()
    return inp, shot, (shot_k, shot_v, shot_i, shot_idx), casc


@pytest.mark.parametrize("name", ["tiny", "llama_reduced", "batch2_group5"])
def test_cascade_equals_one_shot(cake, name):
    cfg = {"tiny": CONFIGS[1],
           "llama_reduced": CONFIGS[2].scaled(n_layers=6, seq_len=2048 + 32 + 9, total_budget=6 * 300),
           "batch2_group5": CONFIGS[5].scaled(n_layers=4, batch=2, seq_len=1300, total_budget=4 * 200)}[name]
    say(f"cascade vs one-shot: {name}")
    inp, shot, (shot_k, shot_v, shot_i, shot_idx), casc = _run_both(cake, cfg)
    L, B, S_w = cfg.n_layers, cfg.batch, cfg.window
    # a layer scored alone gives the same bits as when it is scored in a batch of layers
    np.testing.assert_array_equal(casc.pref, shot.pref)
    np.testing.assert_array_equal(casc.budgets, shot.budgets)
    np.testing.assert_array_equal(casc.keep, shot.keep)
    for m, stage in enumerate(casc.stage_budgets):
        for b in range(B):
            assert list(stage[:, b]) == co.cascade_allocate(casc.pref[b, : m + 1], cfg.total_budget, S_w, cfg.seq_len)
        if m:
            assert np.all(stage[:m] <= casc.stage_budgets[m - 1])            # Prop. 1
    for l in range(L):
        for b in range(B):
            n_k = int(shot.keep[l, b])
            assert torch.equal(casc.idx[l][b, :, :n_k], shot_idx[l][b, :, :n_k])
            assert torch.equal(casc.k_out[l][b, :, : n_k + S_w], shot_k[l][b, :, : n_k + S_w])
            assert torch.equal(casc.v_out[l][b, :, : n_k + S_w], shot_v[l][b, :, : n_k + S_w])
            assert torch.equal(casc.ind_out[l][b, :, :n_k], shot_i[l][b, :, :n_k])
    # the oracle's Alg. 1 on the GPU's indicators and preferences retains the same positions
    if B == 1:
        inds = [shot.indicator[l][0].double().cpu().numpy() for l in range(L)]
        ks = [inp["k"][l, 0].float().cpu().numpy() for l in range(L)]
        vs = [inp["v"][l, 0].float().cpu().numpy() for l in range(L)]
        history, cache = co.cascade_manage(list(casc.pref[0]), inds, ks, vs, cfg.total_budget, S_w)
        assert [list(h) for h in history] == [list(s[:, 0]) for s in casc.stage_budgets]
        for l in range(L):
            n_k = int(casc.keep[l, 0])
            for g in range(cfg.n_kv_heads):
                np.testing.assert_array_equal(casc.idx[l][0, g, :n_k].cpu().numpy(), cache[l]["pos"][g])
                np.testing.assert_array_equal(casc.k_out[l][0, g, : n_k + S_w].float().cpu().numpy(), cache[l]["k"][g])


def test_streaming_session_holds_the_budget_after_every_stage(cake):
    # layers are generated, admitted and released one at a time, as a prefill would produce them
    from synth import make_layer
    cfg = CONFIGS[2].scaled(n_layers=6, seq_len=2048 + 32 + 9, total_budget=6 * 300)
    say("cascade: streaming session")
    session = cake.CascadeSession(cfg.n_layers, cfg.total_budget)
    for l in range(cfg.n_layers):
        one = make_layer(cfg, l, 0, device=DEV)
        stage = session.admit(one["q_win"][None], one["k"][None], one["v"][None])
        del one
        assert stage.shape == (l + 1, 1) and stage.sum() == min(cfg.total_budget, (l + 1) * cfg.seq_len)
        assert session.rows_held() == stage.sum()                 # B = 1: exactly the budget, window rows included
    streamed = session.result()
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    args = ([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)], [inp["v"][l] for l in range(L)])
    batch = cake.EvictionPass(*args, cfg.total_budget).run_cascade()
    np.testing.assert_array_equal(streamed.budgets, batch.budgets)
    np.testing.assert_array_equal(streamed.pref, batch.pref)
    np.testing.assert_array_equal(streamed.keep, batch.keep)
    for l in range(L):
        n_k = int(batch.keep[l, 0])
        assert torch.equal(streamed.k_out[l], batch.k_out[l]) and torch.equal(streamed.v_out[l], batch.v_out[l])
        assert torch.equal(streamed.idx[l][..., :n_k], batch.idx[l][..., :n_k])
        assert torch.equal(streamed.ind_out[l][..., :n_k], batch.ind_out[l][..., :n_k])


def test_cascade_with_handed_over_row_lse_equals_one_shot(cake):
    from gpu_util import torch_row_lse
    cfg = CONFIGS[2].scaled(n_layers=4, seq_len=1500, total_budget=4 * 250)
    say("cascade with handed-over LSE")
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    q = [inp["q_win"][l] for l in range(L)]
    k = [inp["k"][l] for l in range(L)]
    v = [inp["v"][l] for l in range(L)]
    lse = [torch_row_lse(q[l], k[l]) for l in range(L)]
    shot = cake.EvictionPass(q, k, v, cfg.total_budget, row_lse=lse).run()
    torch.cuda.synchronize()
    shot_k = [t.clone() for t in shot.k_out]
    shot_idx = [t.clone() for t in shot.idx]
    casc = cake.EvictionPass(q, k, v, cfg.total_budget, row_lse=lse).run_cascade()
    np.testing.assert_array_equal(casc.budgets, shot.budgets)
    for l in range(L):
        n_k = int(shot.keep[l, 0])
        assert torch.equal(casc.idx[l][0, :, :n_k], shot_idx[l][0, :, :n_k])
        assert torch.equal(casc.k_out[l][0, :, : n_k + cfg.window], shot_k[l][0, :, : n_k + cfg.window])


@pytest.mark.parametrize("name", ["tiny", "llama_reduced", "window64", "everything_fits_at_first", "batch3_group5"])
def test_device_cascade_equals_host_cascade_and_one_shot(cake, name):
    """DeviceCascade (stages chained on the device: plan over the layers seen so far, earlier layers
    re-evicted from their compacted caches with strides taken from the plan) against the host-driven
    CascadeSession stage by stage in the end result, and against the one-shot pass (Thm. 2)."""
    cfg = {"tiny": CONFIGS[1],
           "llama_reduced": CONFIGS[2].scaled(n_layers=6, seq_len=2048 + 32 + 9, total_budget=6 * 300),
           "window64": CONFIGS[4].scaled(n_layers=5, seq_len=4096 + 64 + 3, total_budget=5 * 500),
           "everything_fits_at_first": CONFIGS[2].scaled(n_layers=6, seq_len=700, total_budget=2 * 700 + 333),
           "batch3_group5": CONFIGS[5].scaled(n_layers=4, batch=3, seq_len=1300, total_budget=4 * 200)}[name]
    say(f"device cascade {name}")
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    q = [inp["q_win"][l] for l in range(L)]
    k = [inp["k"][l] for l in range(L)]
    v = [inp["v"][l] for l in range(L)]
    host = cake.CascadeSession(L, cfg.total_budget, track_positions=False)
    dev = cake.DeviceCascade(L, cfg.total_budget)
    for l in range(L):
        host.admit(q[l], k[l], v[l])
        dev.admit(q[l], k[l], v[l])
    want, got = host.result(), dev.result()
    shot = cake.EvictionPass(q, k, v, cfg.total_budget).run()
    torch.cuda.synchronize()
    assert np.array_equal(got.budgets, want.budgets) and np.array_equal(got.keep, want.keep)
    assert np.array_equal(got.budgets, shot.budgets)
    np.testing.assert_array_equal(got.pref, want.pref)
    for l in range(L):
        for s_ in range(cfg.batch):
            n_k = int(want.keep[l, s_])
            for a, b, c in ((got.k_out, want.k_out, shot.k_out), (got.v_out, want.v_out, shot.v_out)):
                assert torch.equal(a[l][s_, :, : n_k + cfg.window], b[l][s_, :, : n_k + cfg.window]), (l, s_, "vs host cascade")
                assert torch.equal(a[l][s_, :, : n_k + cfg.window], c[l][s_, :, : n_k + cfg.window]), (l, s_, "vs one-shot")
            assert torch.equal(got.ind_out[l][s_, :, :n_k], want.ind_out[l][s_, :, :n_k])
            assert torch.equal(got.ind_out[l][s_, :, :n_k], shot.ind_out[l][s_, :, :n_k])
