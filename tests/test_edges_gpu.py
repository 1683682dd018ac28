"""GPU edge cases of the whole pass: nothing to evict, the shortest prefixes, tile boundaries,
a layer that keeps only its window.  Every check is against the oracle on the same tensors."""
import numpy as np
import pytest
import torch

from oracle import cake_oracle as co
from synth import CONFIGS, make_config_inputs

from gpu_util import assert_close, load_cake, oracle_layer, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


def _inputs(cfg):
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    return ([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)], [inp["v"][l] for l in range(L)])


def test_nothing_to_evict_keeps_every_row(cake):
    # B_total >= L*N: every budget is N, the selection is the identity and the caches are copies
    say("edge: nothing to evict")
    cfg = CONFIGS[1].scaled(total_budget=10 ** 6)
    q, k, v = _inputs(cfg)
    res = cake.EvictionPass(q, k, v, cfg.total_budget).run()
    torch.cuda.synchronize()
    assert np.all(res.budgets == cfg.seq_len) and np.all(res.keep == cfg.prefix_len)
    for l in range(cfg.n_layers):
        want = torch.arange(cfg.prefix_len, dtype=torch.int32, device=DEV).expand_as(res.idx[l])
        assert torch.equal(res.idx[l], want)
        assert torch.equal(res.k_out[l], k[l]) and torch.equal(res.v_out[l], v[l])
        assert torch.equal(res.ind_out[l], res.indicator[l])


@pytest.mark.parametrize("n_p", [1, 2, 31, 32, 33, 63, 64, 65, 127, 129])
def test_short_prefixes_and_tile_boundaries(cake, n_p):
    say(f"edge: prefix of {n_p}")
    gen = torch.Generator().manual_seed(100 + n_p)
    #        dtype           d    H_q H_kv S_w  B  L
    for dtype, d, h_q, h_kv, window, B, L in ((torch.float32, 64, 4, 2, 32, 1, 2),
                                              (torch.bfloat16, 128, 8, 2, 32, 2, 2),
                                              (torch.bfloat16, 128, 4, 1, 64, 1, 1),
                                              (torch.bfloat16, 64, 5, 1, 64, 1, 1)):
        N = window + n_p
        q = [(torch.randn(B, h_q, window, d, generator=gen) * 2).to(dtype).to(DEV) for _ in range(L)]
        k = [torch.randn(B, h_kv, N, d, generator=gen).to(dtype).to(DEV) for _ in range(L)]
        v = [torch.randn(B, h_kv, N, d, generator=gen).to(dtype).to(DEV) for _ in range(L)]
        total = L * (window + max(n_p // 2, 1))
        ev = cake.EvictionPass(q, k, v, total)
        res = ev.run()
        torch.cuda.synchronize()
        for l in range(L):
            for b in range(B):
                o = oracle_layer(q[l][b], k[l][b], ev.params)
                assert_close(res.indicator[l][b].cpu().numpy(), o["indicator"], f"indicator n_p={n_p} l={l}")
                assert_close(res.hv[b, l, 0], o["H"], "H")
                assert_close(res.hv[b, l, 1], o["V"], "V")
                n_k = int(res.keep[l, b])
                for g in range(h_kv):
                    got = res.idx[l][b, g, :n_k].cpu().numpy()
                    np.testing.assert_array_equal(got, co.select_topk(res.indicator[l][b, g].double().cpu().numpy(), n_k))
                    np.testing.assert_array_equal(res.k_out[l][b, g, : n_k + window].float().cpu().numpy(),
                                                  co.compact(k[l][b, g].float().cpu().numpy(), got, window))
        for b in range(B):
            assert list(res.budgets[:, b]) == co.cascade_allocate(res.pref[b], total, window, N)
            assert res.budgets[:, b].sum() == min(total, L * N)


def test_layer_without_shift_keeps_only_its_window(cake):
    # Layer 0 attends statically (identical window queries, invisible window keys): V_0 ~ 0, so its
    # preference vanishes next to layer 1's, its budget is the floor S_w and no prefix row survives.
    say("edge: window-only layer")
    torch.manual_seed(11)
    S_w, N, d, H = 32, 800, 64, 2
    q0 = torch.randn(1, H, 1, d, device=DEV).expand(1, H, S_w, d).contiguous()
    k0 = torch.randn(1, H, N, d, device=DEV)
    k0[:, :, N - S_w:, :] = 0
    k0[:, :, N - S_w:, 0] = -1e4 * torch.sign(q0[:, :, :1, 0])
    q1 = torch.randn(1, H, S_w, d, device=DEV) * 3
    k1 = torch.randn(1, H, N, d, device=DEV)
    v0, v1 = torch.randn_like(k0), torch.randn_like(k1)
    total = 2 * S_w + 100
    res = cake.EvictionPass([q0, q1], [k0, k1], [v0, v1], total).run()
    torch.cuda.synchronize()
    assert list(res.budgets[:, 0]) == co.cascade_allocate(res.pref[0], total, S_w, N)
    assert res.budgets[0, 0] == S_w and res.keep[0, 0] == 0 and res.budgets[1, 0] == S_w + 100
    assert torch.equal(res.k_out[0][:, :, :S_w], k0[:, :, N - S_w:]) and torch.equal(res.v_out[0][:, :, :S_w], v0[:, :, N - S_w:])
