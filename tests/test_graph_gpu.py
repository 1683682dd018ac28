"""The one-shot pass under HIP graph capture: scores, preference, device plan, top-k and compaction
are nine launches with no host dependence, so a caller can capture them once and replay.  Every
replay must reproduce the eager result bit for bit, with eager work and synchronisations between
the replays."""
import pytest
import torch

from synth import CONFIGS, make_config_inputs

from gpu_util import load_cake, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


@pytest.mark.parametrize("cid,over", [(2, dict(n_layers=3, seq_len=2048 + 96, total_budget=3 * 300)),
                                      (5, dict(n_layers=2, batch=2, seq_len=1024 + 17, total_budget=2 * 200))])
def test_captured_pass_replays_to_the_eager_result(cake, cid, over):
    cfg = CONFIGS[cid].scaled(**over)
    say(f"graph capture of the one-shot pass: config {cid} {over}")
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    args = ([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)], [inp["v"][l] for l in range(L)])
    eager = cake.EvictionPass(*args, cfg.total_budget)
    want = eager.run()
    torch.cuda.synchronize()
    want_plan = eager.plan.clone()
    want_pools = [t.clone() for t in (eager.pool_k, eager.pool_v, eager.pool_idx, eager.pool_ind)]
    want_ind = eager.indicator.clone()

    ep = cake.EvictionPass(*args, cfg.total_budget)
    ep.scores(); ep.plan_and_evict()                    # warm-up outside the capture (first-use set-up of the kernels)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ep.scores()
            ep.plan_and_evict()
    torch.cuda.current_stream().wait_stream(side)
    n_rows = int(want.keep.sum())
    assert n_rows > 0
    for replay in range(3):
        for t in (ep.pool_k, ep.pool_v, ep.pool_ind, ep.indicator):
            t.zero_()                                   # eager work between the replays; results must come from the replay
        ep.pool_idx.zero_()
        ep.plan.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ep.indicator, want_ind), replay
        budgets, keep, _, _ = ep.read_plan()
        assert (budgets == want.budgets).all() and (keep == want.keep).all()
        caps, off_kv, off_i = ep._placement(keep)
        idx, k_out, v_out, ind_out = ep._views(caps, off_kv, off_i)
        for l in range(L):
            for b in range(cfg.batch):
                n_k = int(keep[l, b])
                assert torch.equal(k_out[l][b, :, : n_k + cfg.window], want.k_out[l][b, :, : n_k + cfg.window]), (replay, l, b)
                assert torch.equal(v_out[l][b, :, : n_k + cfg.window], want.v_out[l][b, :, : n_k + cfg.window])
                assert torch.equal(idx[l][b, :, :n_k], want.idx[l][b, :, :n_k])
                assert torch.equal(ind_out[l][b, :, :n_k], want.ind_out[l][b, :, :n_k])
    del want_plan, want_pools
