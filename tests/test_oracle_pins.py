"""Pins for the CPU oracle: every function is checked against something other than itself.

Hand-derived rationals, closed forms, library routines on special cases, brute force on
tiny inputs and the invariants the paper states (Prop. 1, Thm. 2, budgets summing to B_total).
"""
import itertools
import json
import math
import os
import statistics
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import cake_oracle as co
from synth import CONFIGS, make_layer

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rational_example.json")


def _f(s):
    return float(Fraction(s))


# ---------------------------------------------------------------- worked rational example
def _example_inputs(heads):
    g = json.load(open(GOLDEN))
    k = np.log(np.array(g["keys_exp"], dtype=np.float64)).reshape(1, 4, 1)
    q = np.array([g[h]["q"] for h in heads], dtype=np.float64).reshape(len(heads), 2, 1)
    return g, q, k


@pytest.mark.parametrize("head", ["head0", "head1"])
def test_worked_example_single_head(head):
    g, q, k = _example_inputs([head])
    a = co.window_attention(q, k, scale=1.0)
    # causal mask inside the window: row 0 (position 2) must not see key 3
    assert a[0, 0, 3] == 0.0 and a[0, 1, 3] > 0.0
    a_obs = co.observed(a, 2)
    want = np.array([[_f(x) for x in row] for row in g[head]["a_obs"]])
    np.testing.assert_allclose(a_obs[0], want, rtol=1e-14)
    np.testing.assert_allclose(co.column_variance(a_obs, 1)[0], [_f(x) for x in g[head]["var_unbiased"]], rtol=1e-13)
    np.testing.assert_allclose(co.column_variance(a_obs, 0)[0], [_f(x) / 2 for x in g[head]["var_unbiased"]], rtol=1e-13)
    np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1)[0], [_f(x) for x in g[head]["indicator_gamma200"]], rtol=1e-13)
    np.testing.assert_allclose(co.shift(a_obs, 1)[0], _f(g[head]["V"]), rtol=1e-13)
    h_want = sum(_f(c) * math.log(_f(arg)) for c, arg in g[head]["H_terms"])
    np.testing.assert_allclose(co.dispersion(a_obs)[0], h_want, rtol=1e-13)


def test_worked_example_gqa_pool_and_preference():
    g, q, k = _example_inputs(["head0", "head1"])          # two query heads on one KV head
    p = co.OracleParams(scale=1.0, gamma=200.0, tau1=1.0, tau2=1.0, var_correction=1, pool_kernel=1)
    out = co.layer_pass(q, k, p)
    i0 = [Fraction(x) for x in g["head0"]["indicator_gamma200"]]
    i1 = [Fraction(x) for x in g["head1"]["indicator_gamma200"]]
    want = [float((a + b) / 2) for a, b in zip(i0, i1)]
    np.testing.assert_allclose(out["indicator"][0], want, rtol=1e-13)
    h = [sum(_f(c) * math.log(_f(arg)) for c, arg in g[hd]["H_terms"]) for hd in ("head0", "head1")]
    v = [_f(g[hd]["V"]) for hd in ("head0", "head1")]
    np.testing.assert_allclose(out["H"], (h[0] + h[1]) / 2, rtol=1e-13)
    np.testing.assert_allclose(out["V"], (v[0] + v[1]) / 2, rtol=1e-13)
    np.testing.assert_allclose(out["pref"], (h[0] + h[1]) / 2 * (v[0] + v[1]) / 2, rtol=1e-13)
    # tau exponents of Eq. (6)
    p2 = co.OracleParams(scale=1.0, tau1=0.5, tau2=2.0, pool_kernel=1)
    out2 = co.layer_pass(q, k, p2)
    np.testing.assert_allclose(out2["pref"], ((h[0] + h[1]) / 2) ** 2 * math.sqrt((v[0] + v[1]) / 2), rtol=1e-13)
    # pooling with width 3 over two columns: both become the larger one
    p3 = co.OracleParams(scale=1.0, pool_kernel=3)
    np.testing.assert_allclose(co.layer_pass(q, k, p3)["indicator"][0], [max(want)] * 2, rtol=1e-13)


@pytest.mark.parametrize("head", ["head0", "head1"])
def test_worked_example_indicator_ablation_modes(head):
    """Indicator ablation (Mean, Var, Mean*Var beside Mean + gamma*Var): each mode against the
    rationals of the worked example, and the GQA mean taken on the per-head values."""
    g, q, k = _example_inputs([head])
    a_obs = co.observed(co.window_attention(q, k, scale=1.0), 2)
    mean = [Fraction(x) for x in g[head]["mean"]]
    var = [Fraction(x) for x in g[head]["var_unbiased"]]
    np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1, mode=1)[0], [float(m) for m in mean], rtol=1e-13)
    np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1, mode=2)[0], [float(v) for v in var], rtol=1e-13)
    np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1, mode=3)[0],
                               [float(m * v) for m, v in zip(mean, var)], rtol=1e-13)
    np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1, mode=0)[0],
                               [float(m + 200 * v) for m, v in zip(mean, var)], rtol=1e-13)
    with pytest.raises(ValueError):
        co.head_indicator(a_obs, 200.0, 1, mode=5)


def test_accumulated_attention_indicator_is_the_window_column_sum():
    """Mode 4 (accumulated attention, Sec. 5.5) over the window: per head the sum of the worked
    example's stored attention entries down each prefix column (exact rationals); S_w times the
    mean-only indicator through the whole layer pass; hence the same selection as mode 1 at
    every k, while a decode step (which adds one attention row) moves it S_w times less."""
    g, q, k = _example_inputs(["head0", "head1"])
    a_obs = co.observed(co.window_attention(q, k, scale=1.0), 2)
    for i, head in enumerate(("head0", "head1")):
        rows = [[Fraction(x) for x in row] for row in g[head]["a_obs"]]
        want = [float(sum(col)) for col in zip(*rows)]
        np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1, mode=4)[i], want, rtol=1e-14)
    rng = np.random.default_rng(11)
    q = rng.standard_normal((4, 8, 16)) * 2
    k = rng.standard_normal((2, 90, 16))
    p1 = co.OracleParams(pool_kernel=5, indicator_mode=1)
    p4 = co.OracleParams(pool_kernel=5, indicator_mode=4)
    i1, i4 = co.layer_pass(q, k, p1)["indicator"], co.layer_pass(q, k, p4)["indicator"]
    np.testing.assert_allclose(i4, 8 * i1, rtol=1e-14)
    # brute force: softmax over the visible keys written out, summed down the window rows
    n_p = 90 - 8
    for h in range(4):
        acc = np.zeros(n_p)
        for r in range(8):
            z = (q[h, r] @ k[h // 2, : n_p + r + 1].T) / 4.0
            w = np.exp(z - z.max())
            acc += (w / w.sum())[:n_p]
        np.testing.assert_allclose(co.head_indicator(co.observed(co.window_attention(q, k), 8), 0.0, 1, mode=4)[h], acc, rtol=1e-12)
    for kk in (0, 1, 7, 40, n_p):
        for gi in range(2):
            np.testing.assert_array_equal(co.select_topk(i4[gi], kk), co.select_topk(i1[gi], kk))


def test_indicator_modes_through_layer_pass():
    g, q, k = _example_inputs(["head0", "head1"])
    m = [[Fraction(x) for x in g[h]["mean"]] for h in ("head0", "head1")]
    v = [[Fraction(x) for x in g[h]["var_unbiased"]] for h in ("head0", "head1")]
    want = {1: [(m[0][j] + m[1][j]) / 2 for j in range(2)],
            2: [(v[0][j] + v[1][j]) / 2 for j in range(2)],
            3: [(m[0][j] * v[0][j] + m[1][j] * v[1][j]) / 2 for j in range(2)]}   # product per head, then the group mean
    for mode, w in want.items():
        p = co.OracleParams(scale=1.0, pool_kernel=1, indicator_mode=mode)
        np.testing.assert_allclose(co.layer_pass(q, k, p)["indicator"][0], [float(x) for x in w], rtol=1e-13)
    # the mean-only mode is what gamma = 0 gives in Eq. (11)
    p0 = co.OracleParams(scale=1.0, gamma=0.0, pool_kernel=1)
    p1 = co.OracleParams(scale=1.0, pool_kernel=1, indicator_mode=1)
    np.testing.assert_array_equal(co.layer_pass(q, k, p0)["indicator"], co.layer_pass(q, k, p1)["indicator"])


def test_supplied_row_lse_reproduces_the_worked_example_and_scipy():
    """Window attention from a handed-over log-sum-exp: the rationals of the worked example with
    lse = ln 6, ln 30 (head 0) and ln 14, ln 10 (head 1); scipy's logsumexp on random inputs; and a
    shifted lse scales every weight of that row by exp(-shift)."""
    g, q, k = _example_inputs(["head0", "head1"])
    lse = np.log(np.array([[6.0, 30.0], [14.0, 10.0]]))
    a = co.window_attention_given_lse(q, k, lse, scale=1.0)
    for i, head in enumerate(("head0", "head1")):
        want = np.array([[_f(x) for x in row] for row in g[head]["a_obs"]])
        np.testing.assert_allclose(co.observed(a, 2)[i], want, rtol=1e-14)
    assert a[0, 0, 3] == 0.0                                   # hidden key keeps weight 0
    rng = np.random.default_rng(7)
    q = rng.standard_normal((4, 8, 16)) * 2
    k = rng.standard_normal((2, 60, 16))
    s = co.window_logits(q, k)
    lse = scipy.special.logsumexp(s, axis=-1)
    np.testing.assert_allclose(co.window_attention_given_lse(q, k, lse), co.window_attention(q, k), rtol=1e-12, atol=0)
    p = co.OracleParams(pool_kernel=3)
    a1, a2 = co.layer_pass(q, k, p), co.layer_pass(q, k, p, row_lse=lse)
    np.testing.assert_allclose(a2["indicator"], a1["indicator"], rtol=1e-11)
    np.testing.assert_allclose([a2["H"], a2["V"], a2["pref"]], [a1["H"], a1["V"], a1["pref"]], rtol=1e-11)
    shifted = co.window_attention_given_lse(q, k, lse + 0.5)
    np.testing.assert_allclose(shifted, co.window_attention(q, k) * math.exp(-0.5), rtol=1e-12)


# ---------------------------------------------------------------- softmax
def test_softmax_rows_sum_to_one_and_match_scipy():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((4, 8, 16))
    k = rng.standard_normal((2, 50, 16))
    s = co.window_logits(q, k)
    a = co.softmax_rows(s)
    np.testing.assert_allclose(a.sum(-1), 1.0, atol=1e-12)
    np.testing.assert_allclose(a, scipy.special.softmax(s, axis=-1), rtol=1e-12, atol=0)
    # causal triangle over the last S_w keys: row r sees keys up to N_p + r
    n_p = 50 - 8
    for r in range(8):
        assert np.all(a[:, r, n_p + r + 1:] == 0.0)
        assert np.all(a[:, r, : n_p + r + 1] > 0.0)
    # logits: head h reads KV head h // G, scaled by 1/sqrt(d)
    want = np.einsum("c,c->", q[3, 2], k[1, 7]) / 4.0
    np.testing.assert_allclose(s[3, 2, 7], want, rtol=1e-13)
    # agrees with torch's softmax on the masked logits
    ta = torch.softmax(torch.from_numpy(s), dim=-1).numpy()
    np.testing.assert_allclose(a, ta, rtol=1e-12)


# ---------------------------------------------------------------- closed forms: uniform attention
def test_zero_queries_closed_forms():
    h_q, h_kv, s_w, n, d = 2, 1, 6, 40, 8
    n_p = n - s_w
    q = np.zeros((h_q, s_w, d))
    k = np.random.default_rng(1).standard_normal((h_kv, n, d))
    a_obs = co.observed(co.window_attention(q, k), s_w)
    n_r = [n_p + r + 1 for r in range(s_w)]
    h_want = sum(n_p * math.log(x) / x for x in n_r)
    np.testing.assert_allclose(co.dispersion(a_obs), [h_want] * h_q, rtol=1e-12)
    var_want = statistics.variance([1.0 / x for x in n_r])          # unbiased
    pvar_want = statistics.pvariance([1.0 / x for x in n_r])        # biased
    np.testing.assert_allclose(co.shift(a_obs, 1), [n_p * var_want] * h_q, rtol=1e-10)
    np.testing.assert_allclose(co.shift(a_obs, 0), [n_p * pvar_want] * h_q, rtol=1e-10)
    mean_want = statistics.fmean([1.0 / x for x in n_r])
    np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1), mean_want + 200.0 * var_want, rtol=1e-10)


def test_variance_matches_numpy():
    a = np.random.default_rng(2).random((3, 9, 31))
    np.testing.assert_allclose(co.column_variance(a, 1), np.var(a, axis=-2, ddof=1), rtol=1e-12)
    np.testing.assert_allclose(co.column_variance(a, 0), np.var(a, axis=-2, ddof=0), rtol=1e-12)


def test_entropy_terms_nonnegative_and_zero_log_zero():
    a = np.array([[[0.0, 0.25, 0.5], [1.0, 0.0, 0.0]]])
    h = co.dispersion(a)
    want = -(0.25 * math.log(0.25) + 0.5 * math.log(0.5))
    np.testing.assert_allclose(h, [want], rtol=1e-14)


# ---------------------------------------------------------------- static attention: no temporal shift
def test_static_attention_has_zero_shift():
    row = np.random.default_rng(3).random(57)
    row /= row.sum() * 1.3
    a_obs = np.broadcast_to(row, (2, 16, 57)).copy()
    # zero up to the rounding of the row sum (a few ulp of the mean, squared)
    assert np.all(co.shift(a_obs, 1) <= 1e-28 * np.sum(row ** 2))
    np.testing.assert_allclose(co.head_indicator(a_obs, 200.0, 1), a_obs[:, 0, :], rtol=1e-14)


def test_static_attention_from_q_and_k():
    # identical window queries, window keys pushed out of sight => identical rows
    rng = np.random.default_rng(4)
    s_w, n, d = 8, 200, 16
    q = np.repeat(rng.standard_normal((2, 1, d)), s_w, axis=1)
    k = rng.standard_normal((1, n, d))
    k[:, n - s_w:, :] = 0.0
    k[:, n - s_w:, 0] = -1e4 * np.sign(q[0, 0, 0])
    q[1] = q[0]
    a_obs = co.observed(co.window_attention(q, k), s_w)
    mu = a_obs.mean(axis=-2)
    assert np.all(co.shift(a_obs, 1) <= 1e-12 * np.sum(mu ** 2, axis=-1))


# ---------------------------------------------------------------- indicator
def test_indicator_reduces_to_window_mean_and_is_linear_in_gamma():
    a_obs = np.random.default_rng(5).random((2, 12, 33)) / 40.0
    p0 = co.OracleParams(gamma=0.0, pool_kernel=1)
    np.testing.assert_allclose(co.eviction_indicator(a_obs, 1, p0), a_obs.mean(axis=-2), rtol=1e-13)
    i200 = co.head_indicator(a_obs, 200.0, 1)
    i0 = co.head_indicator(a_obs, 0.0, 1)
    np.testing.assert_allclose(i200 - i0, 200.0 * np.var(a_obs, axis=-2, ddof=1), rtol=1e-10)


def test_gqa_duplicate_heads_and_identity():
    a_one = np.random.default_rng(6).random((1, 8, 21)) / 30.0
    a_dup = np.repeat(a_one, 4, axis=0)
    p = co.OracleParams(pool_kernel=1)
    np.testing.assert_allclose(co.eviction_indicator(a_dup, 4, p), co.eviction_indicator(a_one, 1, p), rtol=1e-13)
    i_q = np.arange(12, dtype=np.float64).reshape(4, 3)
    np.testing.assert_array_equal(co.group_reduce(i_q, 1), i_q)
    np.testing.assert_allclose(co.group_reduce(i_q, 2), [[1.5, 2.5, 3.5], [7.5, 8.5, 9.5]])


@pytest.mark.parametrize("w", [1, 3, 7, 9])
def test_max_pool_matches_torch(w):
    x = np.random.default_rng(7).random((3, 50))
    want = torch.nn.functional.max_pool1d(torch.from_numpy(x).unsqueeze(0), w, stride=1, padding=w // 2)[0].numpy()
    got = co.max_pool(x, w)
    np.testing.assert_array_equal(got, want)
    assert np.all(got >= x)
    if w == 1:
        np.testing.assert_array_equal(got, x)


# ---------------------------------------------------------------- allocation (Eq. 7 / Eq. 9, Prop. 1)
def _brute_force_alloc(pref, total, window, n):
    """Materialise every priority P_l/(s + 1/2) for seat counts s = window..n-1, take the top R."""
    m1 = len(pref)
    if m1 * n <= total:
        return [n] * m1
    if all(p == 0.0 for p in pref):
        pref = [1.0] * m1
    seats = [(-(pref[l] / (s + 0.5)), l, s) for l in range(m1) for s in range(window, n)]
    seats.sort()
    r = total - m1 * window
    out = [window] * m1
    for _, l, _s in seats[:r]:
        out[l] += 1
    return out


def test_allocation_brute_force_tiny():
    rng = np.random.default_rng(8)
    for _ in range(400):
        m1 = int(rng.integers(1, 5))
        window = int(rng.integers(1, 4))
        n = int(rng.integers(window + 1, 24))
        total = int(rng.integers(m1 * window, 65))
        pref = [float(x) for x in rng.choice([0.0, 0.5, 1.0, 2.0, 3.0, 7.5], size=m1)]
        got = co.cascade_allocate(pref, total, window, n)
        assert got == _brute_force_alloc(pref, total, window, n), (pref, total, window, n)


def test_allocation_invariants():
    rng = np.random.default_rng(9)
    for _ in range(200):
        m1 = int(rng.integers(1, 33))
        window, n = 32, int(rng.integers(200, 5000))
        total = int(rng.integers(m1 * window, m1 * n + 50))
        pref = rng.random(m1) * rng.choice([1.0, 10.0, 1e-3], size=m1)
        b = co.cascade_allocate(pref, total, window, n)
        assert sum(b) == min(total, m1 * n)
        assert all(window <= x <= n for x in b)
        for i, j in itertools.combinations(range(m1), 2):
            if pref[i] >= pref[j]:
                assert b[i] >= b[j]
            if pref[i] <= pref[j]:
                assert b[i] <= b[j]


def test_allocation_tracks_eq7_when_unclamped():
    rng = np.random.default_rng(10)
    for _ in range(50):
        m1 = 8
        pref = 1.0 + rng.random(m1)                  # ratios <= 2: neither floor nor cap binds
        total, window, n = 8 * 1024, 32, 100000
        b = co.cascade_allocate(pref, total, window, n)
        exact = pref / pref.sum() * total
        assert np.max(np.abs(np.array(b) - exact)) <= 1.0


def test_allocation_equal_preferences_split_evenly():
    assert co.cascade_allocate([2.0] * 4, 4 * 300, 32, 5000) == [300] * 4
    b = co.cascade_allocate([2.0] * 4, 4 * 300 + 2, 32, 5000)
    assert sorted(b) == [300, 300, 301, 301] and b[:2] == [301, 301]       # ties to the lower layer
    assert co.cascade_allocate([0.0] * 3, 3 * 100, 32, 5000) == [100] * 3    # all-zero => uniform
    assert co.cascade_allocate([0.0, 1.0], 500, 32, 5000) == [32, 468]        # a zero layer keeps its window
    assert co.cascade_allocate([1.0, 3.0], 10_000, 32, 100) == [100, 100]     # everything fits
    with pytest.raises(ValueError):
        co.cascade_allocate([1.0, 1.0], 63, 32, 100)
    with pytest.raises(ValueError):
        co.cascade_allocate([1.0, float("nan")], 640, 32, 100)
    with pytest.raises(ValueError):
        co.cascade_allocate([1.0, -1.0], 640, 32, 100)


def test_allocation_stage_monotone_prop1():
    rng = np.random.default_rng(11)
    for _ in range(300):
        n_layers = int(rng.integers(2, 9))
        window = int(rng.integers(1, 5))
        n = int(rng.integers(10, 60))
        total = int(rng.integers(n_layers * window, n_layers * n))
        pref = rng.choice([0.25, 0.5, 1.0, 1.0, 2.0, 3.0, 0.0], size=n_layers).astype(float)
        prev = None
        for m in range(n_layers):
            cur = co.cascade_allocate(pref[: m + 1], total, window, n)
            if prev is not None:
                assert all(c <= p for c, p in zip(cur, prev)), (pref, total, window, n, m)
            prev = cur


# ---------------------------------------------------------------- top-k and compaction (Eq. 12)
def test_topk_brute_force_and_ties():
    rng = np.random.default_rng(12)
    for _ in range(200):
        n = int(rng.integers(1, 40))
        x = rng.choice([0.0, 0.1, 0.2, 0.3, 0.5], size=n)        # many ties
        k = int(rng.integers(0, n + 1))
        pairs = sorted(((-x[i], i) for i in range(n)))
        want = sorted(i for _, i in pairs[:k])
        got = co.select_topk(x, k)
        assert list(got) == want
    x = np.array([1.0, 3.0, 3.0, 2.0, 3.0])
    assert list(co.select_topk(x, 2)) == [1, 2]                   # lowest positions among equals
    assert list(co.select_topk(x, 4)) == [1, 2, 3, 4]


def test_topk_matches_torch_as_a_set_when_distinct():
    x = np.random.default_rng(13).permutation(500).astype(np.float64)
    got = co.select_topk(x, 37)
    want = torch.topk(torch.from_numpy(x), 37).indices.numpy()
    assert set(got.tolist()) == set(want.tolist())
    assert np.all(np.diff(got) > 0)


def test_compaction_keeps_selected_rows_then_window():
    rows = np.arange(10 * 3, dtype=np.float64).reshape(10, 3)
    idx = np.array([1, 4, 6])
    out = co.compact(rows, idx, 2)
    np.testing.assert_array_equal(out[:3], rows[idx])
    np.testing.assert_array_equal(out[3:], rows[8:])
    k_hat, v_hat, i_hat, got_idx = co.evict(rows, rows + 100, np.array([5., 1., 7., 7., 0., 2., 9., 3.]), 2 + 3, 2)
    assert list(got_idx) == [2, 3, 6]
    np.testing.assert_array_equal(k_hat, np.concatenate([rows[[2, 3, 6]], rows[8:]]))
    np.testing.assert_array_equal(v_hat, k_hat + 100)
    np.testing.assert_array_equal(i_hat, [7., 7., 9.])


# ---------------------------------------------------------------- whole pass on the Tiny config
@pytest.fixture(scope="module")
def tiny():
    cfg = CONFIGS[1]
    p = co.OracleParams()
    layers = [make_layer(cfg, l, 0) for l in range(cfg.n_layers)]
    outs = [co.layer_pass(x["q_win"].double().numpy(), x["k"].double().numpy(), p) for x in layers]
    return cfg, layers, outs


def test_tiny_preferences_differ_and_heavy_hitters_survive(tiny):
    cfg, layers, outs = tiny
    assert outs[1]["H"] < outs[0]["H"]            # 4x temperature => more peaked rows => lower entropy
    assert outs[0]["pref"] > 0 and outs[1]["pref"] > 0 and outs[0]["pref"] != outs[1]["pref"]
    budgets = co.cascade_allocate([o["pref"] for o in outs], cfg.total_budget, cfg.window, cfg.seq_len)
    assert sum(budgets) == cfg.total_budget and budgets[1] > budgets[0]
    # each planted key (+3 logits for every window query) dominates its pooling neighbourhood:
    # 8 planted keys x 7 pooled positions fit in the top 64
    heavy = layers[0]["meta"]["heavy"][0].numpy()
    for g in range(cfg.n_kv_heads):
        kept = set(co.select_topk(outs[0]["indicator"][g], 64).tolist())
        assert set(heavy.tolist()) <= kept


def test_tiny_cascade_equals_one_shot_thm2(tiny):
    cfg, layers, outs = tiny
    prefs = [o["pref"] for o in outs]
    inds = [o["indicator"] for o in outs]
    ks = [x["k"].double().numpy() for x in layers]
    vs = [x["v"].double().numpy() for x in layers]
    budgets, shot = co.one_shot(prefs, inds, ks, vs, cfg.total_budget, cfg.window)
    history, cache = co.cascade_manage(prefs, inds, ks, vs, cfg.total_budget, cfg.window)
    assert history[-1] == budgets
    assert history[0] == [min(cfg.total_budget, cfg.seq_len)]
    for l in range(cfg.n_layers):
        for g in range(cfg.n_kv_heads):
            np.testing.assert_array_equal(cache[l]["pos"][g], shot[l]["pos"][g])
            np.testing.assert_array_equal(cache[l]["k"][g], shot[l]["k"][g])
            np.testing.assert_array_equal(cache[l]["v"][g], shot[l]["v"][g])
            np.testing.assert_array_equal(cache[l]["ind"][g], shot[l]["ind"][g])
            assert shot[l]["k"][g].shape == (budgets[l], cfg.head_dim)
            np.testing.assert_array_equal(shot[l]["k"][g][-cfg.window:], ks[l][g][-cfg.window:])


def test_cascade_equals_one_shot_many_layers_with_ties():
    # pooled indicators tie heavily at the cut; Thm. 2 must still hold with the (value, position) order
    rng = np.random.default_rng(14)
    n_layers, h_kv, n, window, d = 5, 2, 90, 6, 4
    prefs = list(rng.random(n_layers) + 0.1)
    inds = [co.max_pool(rng.choice([0.1, 0.2, 0.3, 0.4], size=(h_kv, n - window)), 5) for _ in range(n_layers)]
    ks = [rng.standard_normal((h_kv, n, d)) for _ in range(n_layers)]
    vs = [rng.standard_normal((h_kv, n, d)) for _ in range(n_layers)]
    budgets, shot = co.one_shot(prefs, inds, ks, vs, 150, window)
    history, cache = co.cascade_manage(prefs, inds, ks, vs, 150, window)
    assert history[-1] == budgets and sum(budgets) == 150
    for l in range(n_layers):
        for g in range(h_kv):
            np.testing.assert_array_equal(cache[l]["pos"][g], shot[l]["pos"][g])
            np.testing.assert_array_equal(cache[l]["k"][g], shot[l]["k"][g])


# ---------------------------------------------------------------- decode-phase maintenance
def test_decode_update_uniform_and_scipy():
    """q = 0 gives weight 1/n to every cached row: the indicator grows by exactly 1/n everywhere.
    Random inputs: scipy's softmax, numpy's group mean and torch's max-pool written out independently."""
    rng = np.random.default_rng(21)
    h_q, h_kv, d, n, w = 4, 2, 8, 50, 6
    k = rng.standard_normal((h_kv, n, d))
    ind = rng.random((h_kv, n - w))
    p = co.OracleParams(pool_kernel=3)
    np.testing.assert_allclose(co.decode_update(np.zeros((h_q, d)), k, ind, w, p), ind + 1.0 / n, rtol=1e-13)
    q = rng.standard_normal((h_q, d)) * 2
    got = co.decode_update(q, k, ind, w, p)
    logits = np.stack([k[h // 2] @ q[h] for h in range(h_q)]) / math.sqrt(d)
    a = scipy.special.softmax(logits, axis=-1)[:, : n - w]
    per_kv = np.stack([a[0:2].mean(0), a[2:4].mean(0)])
    pooled = torch.nn.functional.max_pool1d(torch.from_numpy(per_kv)[None], 3, 1, 1)[0].numpy()
    np.testing.assert_allclose(got, ind + pooled, rtol=1e-12)
    # the weights the new token gives to the window rows are not observed: they only take mass away
    assert np.all(got - ind <= 1.0) and (got - ind).sum() < h_kv * 3.0


def test_decode_step_keeps_the_size_and_evicts_the_lowest():
    rng = np.random.default_rng(22)
    h_q, h_kv, d, cur, w = 2, 1, 4, 10, 3
    cache = {"k": rng.standard_normal((h_kv, cur + w, d)), "v": rng.standard_normal((h_kv, cur + w, d)),
             "ind": np.linspace(0.1, 0.2, cur)[None, :].copy()}
    p = co.OracleParams(pool_kernel=1)
    k_new, v_new = rng.standard_normal((h_kv, d)), rng.standard_normal((h_kv, d))
    out = co.decode_step(np.zeros((h_q, d)), cache, k_new, v_new, w, p)
    assert out["k"].shape == cache["k"].shape and out["ind"].shape == cache["ind"].shape
    # uniform attention adds the same amount everywhere, so the row that just left the window
    # (stored indicator 0) is the one that goes; every older scored row stays in place
    np.testing.assert_array_equal(out["idx"][0], np.arange(cur))
    np.testing.assert_array_equal(out["k"][0, :cur], cache["k"][0, :cur])
    np.testing.assert_array_equal(out["k"][0, cur:], np.concatenate([cache["k"][0, cur + 1:], k_new], axis=0))
    np.testing.assert_allclose(out["ind"][0], cache["ind"][0] + 1.0 / (cur + w + 1), rtol=1e-13)
    # a strong attention to the leaving row keeps it and evicts the weakest old row instead
    cache["k"][0, cur] *= 4.0 / np.linalg.norm(cache["k"][0, cur])          # the longest key by far ...
    q = np.zeros((h_q, d)); q[:] = 10.0 * cache["k"][0, cur]                  # ... and the query points at it
    out = co.decode_step(q, cache, k_new, v_new, w, p)
    assert cur in out["idx"][0] and 0 not in out["idx"][0]


# ---------------------------------------------------------------------------------------------
# Quantised storage of the retained cache (appendix on compatibility with quantisation methods)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantiser_reproduces_grid_values_and_stays_within_half_a_step(bits):
    """Values that already lie on a b-bit grid come back exactly with the codes that built them;
    arbitrary values come back within half a step (plus float32 rounding); codes stay in range;
    a constant group has scale 0, codes 0 and is reproduced exactly."""
    rng = np.random.default_rng(bits)
    levels = 2 ** bits - 1
    codes_in = rng.integers(0, levels + 1, size=(64, 5))
    codes_in[0, :], codes_in[1, :] = 0, levels                      # both ends present in every group of column values
    codes_in[32, :], codes_in[33, :] = 0, levels
    lo, step = np.array([-3.0, 0.5, 10.0, -0.25, 0.0]), np.array([0.5, 0.25, 2.0, 0.125, 1.0])   # exact in float32
    x = lo + codes_in * step
    codes, scale, zero = co.quantize_uniform(x, bits, axis=0)
    np.testing.assert_array_equal(codes, codes_in)
    np.testing.assert_array_equal(zero, np.broadcast_to(lo.astype(np.float32), (2, 5)))
    np.testing.assert_allclose(scale, np.broadcast_to(step, (2, 5)), rtol=1e-6)
    np.testing.assert_allclose(co.dequantize_uniform(codes, scale, zero, 0), x, rtol=1e-6, atol=1e-6)
    y = rng.standard_normal((100, 70)) * 3
    for axis in (0, 1):
        c, s, z = co.quantize_uniform(y, bits, axis=axis)
        assert c.dtype == np.uint8 and c.max() <= levels
        assert s.shape[axis] == -(-y.shape[axis] // 32) and s.shape[1 - axis] == y.shape[1 - axis]
        back = co.dequantize_uniform(c, s, z, axis)
        half = np.repeat(s, 32, axis=axis).take(np.arange(y.shape[axis]), axis=axis) / 2
        assert np.all(np.abs(back - y.astype(np.float32)) <= half * (1 + 1e-5) + 1e-6)
    const = np.full((40, 3), 1.75)
    c, s, z = co.quantize_uniform(const, bits, axis=0)
    assert not c.any() and not s.any() and np.all(z == 1.75)
    np.testing.assert_array_equal(co.dequantize_uniform(c, s, z, 0), const)


def test_quantiser_codes_are_the_nearest_levels_by_brute_force():
    """Every code is the level nearest to its value among all 2^b levels of its group (searched
    exhaustively in float64; values within 1e-6 of a step's midpoint are left out)."""
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((45, 6)) * 2).astype(np.float32)
    for bits in (2, 4):
        c, s, z = co.quantize_uniform(x, bits, axis=0)
        for col in range(x.shape[1]):
            for r in range(x.shape[0]):
                g = r // 32
                grid = float(z[g, col]) + np.arange(2 ** bits) * float(s[g, col])
                d = np.abs(grid - float(x[r, col]))
                best = int(np.argmin(d))
                if np.sort(d)[1] - np.sort(d)[0] > 1e-6:
                    assert c[r, col] == best, (bits, r, col)


def test_quantiser_groups_keys_by_channel_and_values_by_token():
    """Orientation of the two quantisers.  Rows that are all equal (every token the same vector):
    each key channel is constant over tokens, so keys come back exactly, while a value row still
    spreads over its channels and is quantised.  Columns that are all equal (every channel the
    same per token): the other way round.  And a change outside a group leaves the group alone."""
    rng = np.random.default_rng(9)
    row = rng.standard_normal(64).astype(np.float32)
    same_rows = np.tile(row, (50, 1))
    (kc, ks, kz), (vc, vs, vz) = co.quantize_cache(same_rows, same_rows, 4)
    assert ks.shape == (2, 64) and vs.shape == (50, 2)
    assert not ks.any() and np.array_equal(co.dequantize_uniform(kc, ks, kz, 0), same_rows)
    assert vs.all() and np.abs(co.dequantize_uniform(vc, vs, vz, 1) - same_rows).max() > 1e-3
    col = rng.standard_normal(50).astype(np.float32)
    same_cols = np.tile(col[:, None], (1, 64))
    (kc, ks, kz), (vc, vs, vz) = co.quantize_cache(same_cols, same_cols, 4)
    assert not vs.any() and np.array_equal(co.dequantize_uniform(vc, vs, vz, 1), same_cols)
    assert ks.all()
    x = rng.standard_normal((70, 64)).astype(np.float32)
    y = x.copy()
    y[40, 5] += 100.0                                               # token group 1, channel 5 / channel group 0 of token 40
    (kc0, _, _), (vc0, _, _) = co.quantize_cache(x, x, 4)
    (kc1, _, _), (vc1, _, _) = co.quantize_cache(y, y, 4)
    changed_k = np.argwhere(kc0 != kc1)
    assert set(map(tuple, changed_k)) <= {(r, 5) for r in range(32, 64)}
    changed_v = np.argwhere(vc0 != vc1)
    assert set(map(tuple, changed_v)) <= {(40, c) for c in range(0, 32)}
