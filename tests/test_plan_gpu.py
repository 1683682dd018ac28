"""Device-side allocation and planned EVICT (cake_plan_eviction / cake_evict_planned) against the
oracle allocator and against the host-allocated pass: budgets must be identical integers, the
evicted caches identical bits."""
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


def _plan(cake, pref, total, window, seq_len, cur_len=None, h_kv=2, d=64):
    """Budgets and keep counts [L, B] that cake_plan_eviction derives from pref [B, L]."""
    from paper_2503_12491_amd import binding as C
    B, L = pref.shape
    shape = C.make_shape(B, L, h_kv, h_kv, d, seq_len, window, torch.float32)
    plan = torch.zeros(C.cake_plan_bytes(shape), dtype=torch.uint8, device=DEV)
    status = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    pool = torch.zeros(64, dtype=torch.uint8, device=DEV)          # only addresses are derived from the pools here
    cur = None if cur_len is None else torch.tensor(np.asarray(cur_len).reshape(-1), dtype=torch.int32, device=DEV)
    C.cake_plan_eviction(shape, torch.tensor(pref, dtype=torch.float64, device=DEV), total, cur, pool, pool, pool, pool,
                         plan, status)
    torch.cuda.synchronize()
    budgets, keep, cur_out, cap_keep = C.plan_fields(plan.cpu(), L, B)
    assert np.array_equal(cap_keep, keep.max(axis=1))
    return budgets, keep, cur_out, status.cpu().numpy()


def test_device_budgets_equal_the_oracle_allocator(cake):
    rng = np.random.default_rng(7)
    cases = 0
    for trial in range(100):
        L = int(rng.choice([1, 2, 3, 5, 8, 32, 64, 100]))
        B = int(rng.choice([1, 1, 2, 4]))
        window = int(rng.choice([1, 4, 32, 64]))
        seq_len = window + int(rng.integers(1, 1200))
        kind = trial % 6
        pref = rng.random((B, L)) * 10.0 ** rng.integers(-6, 6)
        if kind == 1:
            pref = np.round(pref / pref.max() * 4) / 4             # heavy ties, some exact zeros
        elif kind == 2:
            pref[:, rng.integers(0, L)] = 0.0
        elif kind == 3:
            pref[:] = 0.0                                          # all zero: equal split
        elif kind == 4:
            pref[:, 0] *= 1e6                                      # one layer hits the cap N
        lo = L * window
        total = int(rng.integers(lo, max(lo + 1, L * seq_len + (50 if kind == 5 else -1))))
        budgets, keep, cur, status = _plan(cake, pref, total, window, seq_len)
        assert np.all(status == 0)
        for b in range(B):
            want = co.cascade_allocate(pref[b], total, window, seq_len)
            assert list(budgets[:, b]) == want, (trial, L, B, window, seq_len, total)
            assert list(keep[:, b]) == [min(max(x - window, 0), seq_len - window) for x in want]
        cases += B
    say(f"device allocation: {cases} sequences identical to the oracle allocator")


def test_keep_counts_respect_current_lengths_and_bad_preferences_are_flagged(cake):
    pref = np.array([[1.0, 2.0, 3.0], [0.5, float("nan"), 1.0]])
    cur = np.array([[10, 500], [3, 0], [400, 7]])                  # [L, B]
    budgets, keep, cur_out, status = _plan(cake, pref, 600, 8, 508, cur_len=cur)
    assert list(status) == [0, 1]
    assert np.array_equal(cur_out, cur)
    want0 = co.cascade_allocate(pref[0], 600, 8, 508)
    assert list(budgets[:, 0]) == want0
    assert list(keep[:, 0]) == [min(max(x - 8, 0), c) for x, c in zip(want0, cur[:, 0])]
    # the flagged sequence still gets in-range counts (those of equal preferences)
    assert list(budgets[:, 1]) == co.cascade_allocate([1.0, 1.0, 1.0], 600, 8, 508)
    assert np.all(keep[:, 1] <= cur[:, 1])


@pytest.mark.parametrize("cid,over", [(1, {}), (2, dict(seq_len=2048 + 96, n_layers=5, total_budget=5 * 300)),
                                      (5, dict(seq_len=1024 + 17, n_layers=3, batch=3, total_budget=3 * 200))])
def test_planned_pass_equals_host_allocated_pass(cake, cid, over):
    cfg = CONFIGS[cid].scaled(**over)
    say(f"planned vs host-allocated pass: config {cid} {over}")
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    args = ([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)], [inp["v"][l] for l in range(L)])
    dev_res = cake.EvictionPass(*args, cfg.total_budget).run()
    torch.cuda.synchronize()
    host_res = cake.EvictionPass(*args, cfg.total_budget).run_host_allocated()
    torch.cuda.synchronize()
    assert np.array_equal(dev_res.budgets, host_res.budgets) and np.array_equal(dev_res.keep, host_res.keep)
    assert dev_res.budgets.sum(axis=0).tolist() == [min(cfg.total_budget, L * cfg.seq_len)] * cfg.batch
    for l in range(L):
        for b in range(cfg.batch):
            n_k = int(dev_res.keep[l, b])
            assert torch.equal(dev_res.idx[l][b, :, :n_k], host_res.idx[l][b, :, :n_k])
            assert torch.equal(dev_res.k_out[l][b, :, : n_k + cfg.window], host_res.k_out[l][b, :, : n_k + cfg.window])
            assert torch.equal(dev_res.v_out[l][b, :, : n_k + cfg.window], host_res.v_out[l][b, :, : n_k + cfg.window])
            assert torch.equal(dev_res.ind_out[l][b, :, :n_k], host_res.ind_out[l][b, :, :n_k])
