"""Parity at the full sizes of the benchmark configs, in the launch configuration bench.py times
(all layers resident, one batched pass), on sampled outputs the oracle can compute one by one:
sampled (layer, sequence, KV head) slices for the indicator, one whole layer for H, V and P,
every layer for budgets, sampled rows for top-k and compaction."""
import numpy as np
import pytest
import torch

from oracle import cake_oracle as co
from synth import CONFIGS, make_config_inputs, make_layer

from gpu_util import assert_close, assert_topk_within_ties, load_cake, oracle_layer, oracle_slice, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


def _full_pass(cake, cfg):
    L, B = cfg.n_layers, cfg.batch
    dt = cfg.torch_dtype
    q = torch.empty(L, B, cfg.n_q_heads, cfg.window, cfg.head_dim, dtype=dt, device=DEV)
    k = torch.empty(L, B, cfg.n_kv_heads, cfg.seq_len, cfg.head_dim, dtype=dt, device=DEV)
    v = torch.empty_like(k)
    for l in range(L):
        for b in range(B):
            one = make_layer(cfg, l, b, device=DEV)
            q[l, b], k[l, b], v[l, b] = one["q_win"], one["k"], one["v"]
            del one
    ev = cake.EvictionPass([q[l] for l in range(L)], [k[l] for l in range(L)], [v[l] for l in range(L)],
                           cfg.total_budget)
    res = ev.run()
    torch.cuda.synchronize()
    return q, k, v, ev, res


def _check_sampled(cake, cfg, slices, pref_layers, indicator_slices=()):
    q, k, v, ev, res = _full_pass(cake, cfg)
    L, B, S_w, G = cfg.n_layers, cfg.batch, cfg.window, cfg.group
    params = ev.params
    for b in range(B):
        want = co.cascade_allocate(res.pref[b], cfg.total_budget, S_w, cfg.seq_len)
        assert list(res.budgets[:, b]) == want and sum(want) == cfg.total_budget
    assert np.all(res.pref > 0) and np.all(np.isfinite(res.pref))
    for (l, b) in pref_layers:
        say(f"  whole layer l={l} b={b}")
        o = oracle_layer(q[l, b], k[l, b], params)
        assert_close(res.hv[b, l, 0], o["H"], "H")
        assert_close(res.hv[b, l, 1], o["V"], "V")
        assert_close(res.pref[b, l], o["pref"], "P")
        assert_close(res.indicator[l][b].cpu().numpy(), o["indicator"], "indicator (layer)")
    # always include the slice with the largest budget, so that selection and compaction are
    # exercised on thousands of rows whatever the preferences turn out to be
    l_big, b_big = np.unravel_index(int(np.argmax(res.keep)), res.keep.shape)
    slices = list(slices) + [(int(l_big), int(b_big), min(2, cfg.n_kv_heads - 1))]
    for (l, b, g) in slices:
        say(f"  slice l={l} b={b} g={g}")
        o = oracle_slice(q[l, b], k[l, b], g, G, params)
        gpu_ind = res.indicator[l][b, g].double().cpu().numpy()
        worst = assert_close(gpu_ind, o["indicator"], f"indicator l={l} b={b} g={g}")
        n_k = int(res.keep[l, b])
        got = res.idx[l][b, g, :n_k].cpu().numpy()
        np.testing.assert_array_equal(got, co.select_topk(gpu_ind, n_k))
        assert_topk_within_ties(got, o["indicator"], n_k)
        for src, dst in ((k, res.k_out), (v, res.v_out)):
            rows = src[l, b, g].float().cpu().numpy()
            np.testing.assert_array_equal(dst[l][b, g, : n_k + S_w].float().cpu().numpy(), co.compact(rows, got, S_w))
        np.testing.assert_array_equal(res.ind_out[l][b, g, :n_k].cpu().numpy(), res.indicator[l][b, g].cpu().numpy()[got])
        say(f"    worst indicator error {worst:.2e}, kept {n_k}")
    # further slices for the indicator alone (layers differ in temperature, which drives both the
    # re-referencing of the running sums and the spread of the weights)
    for (l, b, g) in indicator_slices:
        o = oracle_slice(q[l, b], k[l, b], g, G, params)
        worst = assert_close(res.indicator[l][b, g].double().cpu().numpy(), o["indicator"], f"indicator l={l} b={b} g={g}")
        say(f"  indicator slice l={l} b={b} g={g}: worst error {worst:.2e}")
    # properties that hold at any size, on every row
    for l in range(L):
        for b in range(B):
            n_k = int(res.keep[l, b])
            ix = res.idx[l][b, :, :n_k]
            if n_k > 1:
                assert torch.all(ix[:, 1:] > ix[:, :-1])
            if n_k:
                assert int(ix.min()) >= 0 and int(ix.max()) < cfg.prefix_len
            assert torch.equal(res.k_out[l][b, :, n_k: n_k + S_w], k[l, b, :, cfg.prefix_len:])
    del q, k, v, ev, res
    torch.cuda.empty_cache()


def test_config2_llama_8k(cake):
    say("full size: config 2")
    _check_sampled(cake, CONFIGS[2], slices=[(0, 0, 0), (13, 0, 5), (31, 0, 7)], pref_layers=[(3, 0), (16, 0)])


def test_config3_llama_32k_drifting_heavy_hitters(cake):
    say("full size: config 3")
    cfg = CONFIGS[3]
    _check_sampled(cake, cfg, slices=[(2, 0, 1), (30, 0, 6)], pref_layers=[(9, 0)])


def test_config4_llama_128k_bench_configuration(cake):
    say("full size: config 4 (the benchmark workload)")
    # one slice of every layer on top of the fully checked ones
    _check_sampled(cake, CONFIGS[4], slices=[(0, 0, 0), (17, 0, 3), (31, 0, 7)], pref_layers=[(5, 0)],
                   indicator_slices=[(l, 0, (3 * l + 1) % 8) for l in range(32)])


def test_config5_gqa5_batch4(cake):
    say("full size: config 5")
    _check_sampled(cake, CONFIGS[5], slices=[(0, 0, 0), (40, 2, 4), (63, 3, 7)], pref_layers=[(63, 1)])


def test_config2_full_cascade_equals_one_shot(cake):
    # Alg. 1 over all 32 layers at full size: the same caches as the one-shot pass (Thm. 2),
    # budgets never growing from stage to stage (Prop. 1)
    cfg = CONFIGS[2]
    say("full size: config 2 cascade vs one-shot")
    inp = make_config_inputs(cfg, device=DEV)
    L, S_w = cfg.n_layers, cfg.window
    args = ([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)], [inp["v"][l] for l in range(L)])
    shot = cake.EvictionPass(*args, cfg.total_budget).run()
    torch.cuda.synchronize()
    shot_k = [t.clone() for t in shot.k_out]
    shot_idx = [t.clone() for t in shot.idx]
    casc = cake.EvictionPass(*args, cfg.total_budget).run_cascade()
    np.testing.assert_array_equal(casc.budgets, shot.budgets)
    assert casc.budgets.sum() == cfg.total_budget
    for m in range(1, L):
        assert np.all(casc.stage_budgets[m][:m] <= casc.stage_budgets[m - 1])
    for l in range(L):
        n_k = int(shot.keep[l, 0])
        assert torch.equal(casc.idx[l][0, :, :n_k], shot_idx[l][0, :, :n_k])
        assert torch.equal(casc.k_out[l][0, :, : n_k + S_w], shot_k[l][0, :, : n_k + S_w])


def test_half_a_million_keys(cake):
    """Four times the benchmark's context: N = 524288, S_w = 64, one layer, two KV heads of four
    query heads (offsets beyond 2^27 elements per slice, 256 chunks per slice); one slice against
    the oracle, the other by the properties that hold at any size."""
    say("full size: N = 524288")
    cfg = CONFIGS[4].scaled(n_layers=1, n_q_heads=8, n_kv_heads=2, seq_len=524288, total_budget=4096)
    _check_sampled(cake, cfg, slices=[(0, 0, 1)], pref_layers=[])
