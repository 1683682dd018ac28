"""Seeded random small problems through the whole pass (scores, preferences, budgets, top-k,
compaction) against the oracle: group sizes 1..8, both head sizes, both windows, both dtypes,
ragged lengths around the tile and chunk boundaries, batches of 1..3, all indicator modes."""
import numpy as np
import pytest
import torch

from oracle import cake_oracle as co

from gpu_util import assert_close, assert_topk_within_ties, load_cake, oracle_layer, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


def _case(rng):
    group = int(rng.choice([1, 2, 3, 4, 5, 8]))
    h_kv = int(rng.choice([1, 2, 3]))
    d = int(rng.choice([64, 128]))
    window = int(rng.choice([32, 64]))
    dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
    B = int(rng.choice([1, 1, 2, 3]))
    L = int(rng.choice([1, 2, 3]))
    n_p = int(rng.choice([int(rng.integers(1, 40)), int(rng.integers(60, 70)), int(rng.integers(250, 262)),
                          int(rng.integers(500, 530)), int(rng.integers(700, 1100))]))
    N = n_p + window
    frac = rng.choice([0.1, 0.3, 0.8, 2.0])
    total = int(max(L * window + 1, L * (window + frac * n_p)))
    params = dict(gamma=float(rng.choice([0.0, 50.0, 200.0])), pool_kernel=int(rng.choice([1, 3, 7])),
                  var_correction=int(rng.choice([0, 1])), indicator_mode=int(rng.choice([0, 0, 0, 1, 2, 3, 4])),
                  tau1=float(rng.choice([0.5, 1.0, 2.0])), tau2=float(rng.choice([0.5, 1.0, 3.0])))
    return group, h_kv, d, window, dtype, B, L, N, total, params


@pytest.mark.parametrize("seed", range(24))
def test_random_problem(cake, seed):
    rng = np.random.default_rng(1000 + seed)
    group, h_kv, d, window, dtype, B, L, N, total, pk = _case(rng)
    say(f"random {seed}: G={group} H_kv={h_kv} d={d} S_w={window} {dtype} B={B} L={L} N={N} B_total={total} {pk}")
    gen = torch.Generator().manual_seed(seed)
    temp = [float(rng.uniform(0.5, 3.0)) for _ in range(L)]
    q = [(torch.randn(B, group * h_kv, window, d, generator=gen) * temp[l]).to(dtype).to(DEV) for l in range(L)]
    k = [torch.randn(B, h_kv, N, d, generator=gen).to(dtype).to(DEV) for _ in range(L)]
    v = [torch.randn(B, h_kv, N, d, generator=gen).to(dtype).to(DEV) for _ in range(L)]
    params = cake.make_params(**pk)
    ev = cake.EvictionPass(q, k, v, total, params)
    res = ev.run()
    torch.cuda.synchronize()
    for l in range(L):
        for b in range(B):
            o = oracle_layer(q[l][b], k[l][b], params)
            assert_close(res.indicator[l][b].cpu().numpy(), o["indicator"], f"indicator l={l} b={b}")
            assert_close(res.hv[b, l, 0], o["H"], "H")
            assert_close(res.hv[b, l, 1], o["V"], "V")
            n_k = int(res.keep[l, b])
            for g in range(h_kv):
                got = res.idx[l][b, g, :n_k].cpu().numpy()
                np.testing.assert_array_equal(got, co.select_topk(res.indicator[l][b, g].double().cpu().numpy(), n_k))
                np.testing.assert_array_equal(res.k_out[l][b, g, : n_k + window].float().cpu().numpy(),
                                              co.compact(k[l][b, g].float().cpu().numpy(), got, window))
                np.testing.assert_array_equal(res.v_out[l][b, g, : n_k + window].float().cpu().numpy(),
                                              co.compact(v[l][b, g].float().cpu().numpy(), got, window))
    for b in range(B):
        assert list(res.budgets[:, b]) == co.cascade_allocate(res.pref[b], total, window, N)
    # cascade mode ends with the same caches
    casc = cake.EvictionPass(q, k, v, total, params).run_cascade()
    np.testing.assert_array_equal(casc.budgets, res.budgets)
    for l in range(L):
        for b in range(B):
            n_k = int(res.keep[l, b])
            assert torch.equal(casc.k_out[l][b, :, : n_k + window], res.k_out[l][b, :, : n_k + window])
            assert torch.equal(casc.idx[l][b, :, :n_k], res.idx[l][b, :, :n_k])
