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
