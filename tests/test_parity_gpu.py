"""GPU parity: every libcake call against the CPU oracle on the same seeded inputs.

Bars: indicators / H / V / P within 1e-3 relative (bf16 or fp32 inputs, fp32 arithmetic on the
GPU, fp64 in the oracle); budgets exact when the oracle allocator is fed the GPU's preferences;
indices and compacted K/V bit-exact when the oracle's top-k is fed the GPU's indicator.
"""
import numpy as np
import pytest
import torch

from oracle import cake_oracle as co
from synth import CONFIGS, make_config_inputs

from gpu_util import (ATOL, RTOL, assert_close, assert_topk_within_ties, host64, load_cake, oracle_layer, say,
                      torch_row_lse)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


# ------------------------------------------------------------------------------------ compaction
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64), (torch.bfloat16, 64)])
def test_compact_kv_bit_exact(cake, dtype, d):
    say(f"compact dtype={dtype} d={d}")
    torch.manual_seed(1)
    L, B, H, S_w = 3, 2, 2, 32
    cur = [[700, 650], [33, 1], [257, 257]]            # per (layer, sequence) prefix lengths
    keep = [[129, 5], [33, 0], [1, 200]]
    shape = cake.make_shape(B, L, 2 * H, H, d, 1024, S_w, dtype)
    k_in, v_in, ind_in, idx, k_out, v_out, ind_out, strides = [], [], [], [], [], [], [], []
    for l in range(L):
        cap_cur, cap_keep = max(cur[l]), max(keep[l])
        rows = cap_cur + S_w + 5                        # spare rows: strides need not be tight
        k_in.append(torch.randn(B, H, rows, d, device=DEV).to(dtype))
        v_in.append(torch.randn(B, H, rows, d, device=DEV).to(dtype))
        ind_in.append(torch.rand(B, H, cap_cur, device=DEV))
        ix = torch.zeros(B, H, max(cap_keep, 1), dtype=torch.int32, device=DEV)
        for b in range(B):
            for h in range(H):
                if keep[l][b]:
                    sel = torch.randperm(cur[l][b])[: keep[l][b]].sort().values
                    ix[b, h, : keep[l][b]] = sel.to(torch.int32).to(DEV)
        idx.append(ix)
        k_out.append(torch.full((B, H, cap_keep + S_w, d), -7.0, device=DEV).to(dtype))
        v_out.append(torch.full((B, H, cap_keep + S_w, d), -7.0, device=DEV).to(dtype))
        ind_out.append(torch.full((B, H, max(cap_keep, 1)), -7.0, device=DEV))
        strides.append([k_in[l].stride(0), k_in[l].stride(1), k_in[l].stride(2)])
    flat = lambda a: [x for row in a for x in row]
    cake.cake_compact_kv(shape, cake.ptr_table(k_in), cake.ptr_table(v_in), strides, flat(cur), flat(keep),
                         cake.ptr_table(idx), cake.ptr_table(ind_in), cake.ptr_table(k_out),
                         cake.ptr_table(v_out), cake.ptr_table(ind_out))
    torch.cuda.synchronize()
    for l in range(L):
        cap_keep = max(keep[l])
        for b in range(B):
            for h in range(H):
                n_k, n_c = keep[l][b], cur[l][b]
                sel = idx[l][b, h, :n_k].long().cpu().numpy()
                rows_in = k_in[l][b, h, : n_c + S_w].float().cpu().numpy()
                want = co.compact(rows_in, sel, S_w)
                got = k_out[l][b, h, : n_k + S_w].float().cpu().numpy()
                np.testing.assert_array_equal(got, want)
                rows_in = v_in[l][b, h, : n_c + S_w].float().cpu().numpy()
                np.testing.assert_array_equal(v_out[l][b, h, : n_k + S_w].float().cpu().numpy(),
                                              co.compact(rows_in, sel, S_w))
                np.testing.assert_array_equal(ind_out[l][b, h, :n_k].cpu().numpy(),
                                              ind_in[l][b, h].cpu().numpy()[sel])
                # rows past this sequence's count are untouched
                assert torch.all(k_out[l][b, h, n_k + S_w:].float() == -7.0)
                assert torch.all(ind_out[l][b, h, n_k:cap_keep] == -7.0) if cap_keep else True


# ------------------------------------------------------------------------------------ top-k
def _run_topk(cake, rows, cur, keep):
    """rows: list over layers of [B,H,cap] f32 device tensors; cur/keep [L][B]."""
    L, B, H = len(rows), rows[0].shape[0], rows[0].shape[1]
    shape = cake.make_shape(B, L, H, H, 64, 1024, 32, torch.float32)
    idx = [torch.full((B, H, max(max(keep[l]), 1)), -1, dtype=torch.int32, device=DEV) for l in range(L)]
    flat = lambda a: [x for row in a for x in row]
    cake.cake_select_topk(shape, cake.ptr_table(rows), flat(cur), flat(keep), cake.ptr_table(idx))
    torch.cuda.synchronize()
    return idx


def test_select_topk_matches_oracle_with_ties_and_ragged_lengths(cake):
    say("topk ties/ragged")
    g = torch.Generator().manual_seed(2)
    cases = [(1, 1), (1, 0), (5, 5), (5, 2), (1023, 100), (1024, 1024), (4096, 17), (4097, 4096), (4100, 2048),
             (70001, 3333), (131008, 1984)]
    for cur, keep in cases:
        for kind in ("distinct", "ties", "pooled", "zeros"):
            if kind == "distinct":
                x = torch.rand(cur, generator=g) * 1e-3
            elif kind == "ties":
                x = torch.randint(0, 6, (cur,), generator=g).float() * 0.125
            elif kind == "pooled":
                x = torch.nn.functional.max_pool1d(torch.rand(1, cur, generator=g), 7, 1, 3)[0] if cur >= 1 else None
            else:
                x = torch.zeros(cur)
                x[::3] = -0.0
            rows = [x.view(1, 1, cur).to(DEV).contiguous()]
            idx = _run_topk(cake, rows, [[cur]], [[keep]])
            want = co.select_topk(x.double().numpy(), keep)
            np.testing.assert_array_equal(idx[0][0, 0, :keep].cpu().numpy(), want, err_msg=f"{cur} {keep} {kind}")


def test_select_topk_batched_layers_and_negative_values(cake):
    say("topk batched")
    g = torch.Generator().manual_seed(3)
    L, B, H = 3, 2, 3
    cur = [[501, 37], [9003, 9003], [66, 1]]      # row starts fall on all four 16-byte phases
    keep = [[20, 37], [1000, 1], [0, 1]]
    rows = []
    for l in range(L):
        cap = max(cur[l])
        rows.append((torch.randn(B, H, cap, generator=g) * 3).round().div(4).to(DEV))   # negatives and ties
    idx = _run_topk(cake, rows, cur, keep)
    for l in range(L):
        for b in range(B):
            for h in range(H):
                x = rows[l][b, h, : cur[l][b]].double().cpu().numpy()
                np.testing.assert_array_equal(idx[l][b, h, : keep[l][b]].cpu().numpy(), co.select_topk(x, keep[l][b]))


# ------------------------------------------------------------------------------------ scores
def _check_scores(cake, cfg, params=None, layers=None, check_layers=None, handoff=False):
    params = params or cake.make_params()
    inp = make_config_inputs(cfg, device=DEV, layers=layers)
    L = len(inp["layers"])
    q = [inp["q_win"][l] for l in range(L)]
    k = [inp["k"][l] for l in range(L)]
    v = [inp["v"][l] for l in range(L)]
    # handoff: the rows' log-sum-exp comes from outside (here torch), the scores take one pass over K
    lse = [torch_row_lse(q[l], k[l], params.scale) for l in range(L)] if handoff else None
    ev = cake.EvictionPass(q, k, v, cfg.total_budget, params, row_lse=lse)
    ev.scores()
    pref, hv = ev.preferences_to_host()
    ind = ev.indicator.cpu().numpy()
    worst = {}
    for l in (check_layers if check_layers is not None else range(L)):
        for b in range(cfg.batch):
            o = oracle_layer(q[l][b], k[l][b], params, lse[l][b] if handoff else None)
            worst["ind"] = max(worst.get("ind", 0), assert_close(ind[l, b], o["indicator"], f"indicator l={l} b={b}"))
            worst["H"] = max(worst.get("H", 0), assert_close(hv[b, l, 0], o["H"], f"H l={l} b={b}"))
            worst["V"] = max(worst.get("V", 0), assert_close(hv[b, l, 1], o["V"], f"V l={l} b={b}"))
            worst["P"] = max(worst.get("P", 0), assert_close(pref[b, l], o["pref"], f"P l={l} b={b}"))
    say(f"  worst relative errors {worst}")
    return ev, inp


def test_scores_tiny_fp32(cake):
    say("scores tiny fp32")
    _check_scores(cake, CONFIGS[1])


def test_scores_bf16_ragged_chunks(cake):
    # Llama shape, N chosen so that chunks, 64-key tiles and 32-key sub-tiles all end ragged
    say("scores bf16 ragged")
    cfg = CONFIGS[2].scaled(n_layers=2, seq_len=2048 + 777, total_budget=2 * 512)
    _check_scores(cake, cfg)


@pytest.mark.parametrize("h_q,h_kv,d,layers,batch", [
    (10, 2, 128, 1, 1),      # G = 5: two slices in a workgroup of three (one repeats the last slice, stores nothing)
    (20, 4, 64, 1, 1),       # G = 5, d = 64: four slices, two workgroups
    (12, 2, 128, 2, 1),      # G = 6: two slices per workgroup, exactly filled
    (18, 3, 64, 1, 3),       # G = 6, d = 64, batch of 3: nine slices, the last workgroup half empty
])
def test_scores_packed_workgroups_for_groups_of_5_and_6(cake, h_q, h_kv, d, layers, batch):
    """bf16 S_w = 32 kernels that put several (layer, sequence, KV head) slices in one workgroup:
    slice counts that do and do not fill the last workgroup, ragged chunk ends, the tail path."""
    say(f"scores packed H_q={h_q} H_kv={h_kv} d={d} L={layers} B={batch}")
    cfg = CONFIGS[2].scaled(n_q_heads=h_q, n_kv_heads=h_kv, head_dim=d, n_layers=layers, batch=batch,
                            seq_len=512 + 32 + 45, total_budget=layers * 200)
    _check_scores(cake, cfg)
    _check_scores(cake, cfg, cake.make_params(indicator_mode=cake.CAKE_IND_VAR, pool_kernel=3))


def test_scores_window64_and_drifting_heavy_hitters(cake):
    say("scores S_w=64 / drift")
    cfg = CONFIGS[3].scaled(n_layers=2, seq_len=4096 + 64 + 5, window=64, total_budget=2 * 400)
    _check_scores(cake, cfg)


def test_scores_group5_batch2(cake):
    say("scores G=5 batch=2")
    cfg = CONFIGS[5].scaled(n_layers=3, batch=2, seq_len=3000, total_budget=3 * 300)
    _check_scores(cake, cfg)


def test_scores_parameter_variants(cake):
    say("scores params")
    cfg = CONFIGS[2].scaled(n_layers=1, seq_len=1500, total_budget=512, n_q_heads=8, n_kv_heads=8)   # G = 1
    _check_scores(cake, cfg, cake.make_params(scale=0.07, gamma=0.0, tau1=0.5, tau2=2.0, var_correction=0, pool_kernel=1))
    cfg = CONFIGS[1].scaled(head_dim=128, seq_len=600)
    _check_scores(cake, cfg, cake.make_params(gamma=50.0, pool_kernel=3))
    cfg = CONFIGS[2].scaled(n_layers=1, seq_len=1200, head_dim=64, total_budget=512)
    _check_scores(cake, cfg)
    cfg = CONFIGS[1].scaled(head_dim=128, window=64, seq_len=700)          # fp32, two row blocks per wave
    _check_scores(cake, cfg)
    cfg = CONFIGS[1].scaled(window=64, seq_len=450)
    _check_scores(cake, cfg)


def test_scores_pooling_widths_and_row_alignment(cake):
    # the pooling kernel has a 16-byte path (rows of a multiple of four positions, windows up to nine)
    # and a general one; both, on prefixes longer than one pooling span, edges included
    say("scores pooling widths")
    for seq_len in (2048 + 32 + 2072, 2048 + 32 + 2071):          # prefix 4120 (multiple of four) and 4119
        cfg = CONFIGS[2].scaled(n_layers=1, seq_len=seq_len, total_budget=512, n_q_heads=4, n_kv_heads=2)
        for pool in (1, 5, 9, 11, 129):
            _check_scores(cake, cfg, cake.make_params(pool_kernel=pool))


def test_scores_with_handed_over_row_lse(cake):
    # single pass over K with the normalisers supplied: against the oracle fed the same f32 values,
    # and against the library's own two-pass result
    say("scores with handed-over LSE")
    for cfg, params in [(CONFIGS[2].scaled(n_layers=2, seq_len=2048 + 32 + 45, total_budget=2 * 400), None),
                        (CONFIGS[4].scaled(n_layers=1, seq_len=1500, total_budget=300), cake.make_params(scale=0.11, pool_kernel=3)),
                        (CONFIGS[5].scaled(n_layers=2, batch=2, seq_len=1111, total_budget=2 * 200), None),
                        (CONFIGS[1], None)]:
        ev, inp = _check_scores(cake, cfg, params, handoff=True)
        one_pass = ev.indicator.clone()
        pref1, hv1 = ev.preferences_to_host()
        pref1, hv1 = pref1.copy(), hv1.copy()
        two = cake.EvictionPass(ev.q_win, ev.k, ev.v, cfg.total_budget, ev.params)
        two.scores()
        pref2, hv2 = two.preferences_to_host()
        assert_close(one_pass.cpu().numpy(), two.indicator.cpu().numpy(), "one-pass vs two-pass indicator", rtol=2e-4)
        assert_close(hv1, hv2, "one-pass vs two-pass H, V", rtol=2e-4)
        assert_close(pref1, pref2, "one-pass vs two-pass P", rtol=4e-4)


def test_pass_with_handed_over_row_lse(cake):
    say("pass with handed-over LSE")
    cfg = CONFIGS[2].scaled(n_layers=3, seq_len=3000, total_budget=3 * 500)
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    q = [inp["q_win"][l] for l in range(L)]
    k = [inp["k"][l] for l in range(L)]
    v = [inp["v"][l] for l in range(L)]
    lse = [torch_row_lse(q[l], k[l]) for l in range(L)]
    res = cake.EvictionPass(q, k, v, cfg.total_budget, row_lse=lse).run()
    torch.cuda.synchronize()
    for b in range(cfg.batch):
        assert list(res.budgets[:, b]) == co.cascade_allocate(res.pref[b], cfg.total_budget, cfg.window, cfg.seq_len)
    for l in range(L):
        o = oracle_layer(q[l][0], k[l][0], cake.make_params(), lse[l][0])
        n_k = int(res.keep[l, 0])
        for g in range(cfg.n_kv_heads):
            got = res.idx[l][0, g, :n_k].cpu().numpy()
            np.testing.assert_array_equal(got, co.select_topk(res.indicator[l][0, g].double().cpu().numpy(), n_k))
            assert_topk_within_ties(got, o["indicator"][g], n_k)
            np.testing.assert_array_equal(res.k_out[l][0, g, : n_k + cfg.window].float().cpu().numpy(),
                                          co.compact(k[l][0, g].float().cpu().numpy(), got, cfg.window))


def test_scores_static_attention_has_no_shift(cake):
    # identical window queries and invisible window keys: every window row is the same
    # distribution, so V must vanish (up to fp32 cancellation) and I must equal the mean.
    say("scores static attention")
    torch.manual_seed(5)
    S_w, N, d, H = 32, 1000, 64, 2
    q = torch.randn(1, H, 1, d, device=DEV).expand(1, H, S_w, d).contiguous()
    k = torch.randn(1, H, N, d, device=DEV)
    k[:, :, N - S_w:, :] = 0
    k[:, :, N - S_w:, 0] = -1e4 * torch.sign(q[:, :, :1, 0])
    ev = cake.EvictionPass([q], [k], [k.clone()], 256, cake.make_params(pool_kernel=1))
    ev.scores()
    pref, hv = ev.preferences_to_host()
    ind = ev.indicator[0, 0].double().cpu().numpy()
    o = oracle_layer(q[0], k[0], cake.make_params(pool_kernel=1))
    assert_close(ind, o["indicator"], "static indicator")
    mu2 = float(np.sum(o["indicator"] ** 2) / H)
    assert hv[0, 0, 1] <= 1e-5 * mu2, (hv[0, 0, 1], mu2)


def test_scores_one_hot_attention_keeps_preferences_finite(cake):
    # Every window row of layer 0 puts all but ~2^-60 of its weight on one key: the dispersion is
    # of the order of 1e-16 and the fp32 sum behind it is rounding noise of either sign.  It must
    # come out finite and non-negative (never NaN after the powers of Eq. 6), the pass must run,
    # and the budgets must equal the oracle allocator's on the GPU's preferences.
    say("scores one-hot attention")
    torch.manual_seed(8)
    S_w, N, d, H = 32, 600, 64, 2
    q0 = torch.randn(1, H, S_w, d, device=DEV)
    k0 = torch.randn(1, H, N, d, device=DEV) * 0.05
    k0[:, :, 17, :] = 60.0 * q0[:, :, 0, :] / q0[:, :, 0, :].norm(dim=-1, keepdim=True)
    q0 = q0[:, :, :1, :].expand(1, H, S_w, d).contiguous() * 8
    q1 = torch.randn(1, H, S_w, d, device=DEV)
    k1 = torch.randn(1, H, N, d, device=DEV)
    p = cake.make_params(tau1=0.7, tau2=1.3)
    ev = cake.EvictionPass([q0, q1], [k0, k1], [k0.clone(), k1.clone()], 400, p)
    res = ev.run()
    torch.cuda.synchronize()
    assert np.all(np.isfinite(res.pref)) and np.all(res.pref >= 0) and np.all(res.hv >= 0)
    o0 = oracle_layer(q0[0], k0[0], p)
    assert o0["H"] < 1e-6 and abs(res.hv[0, 0, 0] - o0["H"]) <= 1e-3      # noise floor of the fp32 logits
    o1 = oracle_layer(q1[0], k1[0], p)
    assert_close(res.pref[0, 1], o1["pref"], "P of the ordinary layer")
    assert list(res.budgets[:, 0]) == co.cascade_allocate(res.pref[0], 400, S_w, N)
    assert res.budgets[0, 0] < res.budgets[1, 0]


def test_scores_rescale_path_and_large_logits(cake):
    # logits that climb by hundreds of log2 units along the keys force pass 1 to re-reference
    say("scores rescale path")
    torch.manual_seed(6)
    S_w, N, d, H = 32, 700, 64, 2
    q = torch.randn(1, H, S_w, d, device=DEV)
    k = torch.randn(1, H, N, d, device=DEV)
    ramp = torch.linspace(0, 1, N, device=DEV).view(1, 1, N, 1)
    k = k + 60.0 * ramp * q[:, :, :1, :] / q[:, :, :1, :].norm(dim=-1, keepdim=True)
    p = cake.make_params(pool_kernel=1)
    ev = cake.EvictionPass([q], [k], [k.clone()], 256, p)
    ev.scores()
    pref, hv = ev.preferences_to_host()
    o = oracle_layer(q[0], k[0], p)
    assert_close(ev.indicator[0, 0].cpu().numpy(), o["indicator"], "ramp indicator")
    assert_close(hv[0, 0, 0], o["H"], "ramp H")


# ------------------------------------------------------------------------------------ whole pass
def _check_pass(cake, cfg, params=None):
    params = params or cake.make_params()
    ev, inp = _check_scores(cake, cfg, params)
    res = ev.run()
    torch.cuda.synchronize()
    L, B, S_w = cfg.n_layers, cfg.batch, cfg.window
    for b in range(B):
        want = co.cascade_allocate(res.pref[b], cfg.total_budget, S_w, cfg.seq_len)
        assert list(res.budgets[:, b]) == want                      # exact, fed the GPU's preferences
        assert sum(want) == min(cfg.total_budget, L * cfg.seq_len)
    swaps = 0
    for l in range(L):
        for b in range(B):
            n_k = int(res.keep[l, b])
            o = oracle_layer(inp["q_win"][l][b], inp["k"][l][b], params)
            for g in range(cfg.n_kv_heads):
                gpu_ind = res.indicator[l][b, g].double().cpu().numpy()
                got = res.idx[l][b, g, :n_k].cpu().numpy()
                np.testing.assert_array_equal(got, co.select_topk(gpu_ind, n_k))     # bit-exact on GPU indicator
                swaps += assert_topk_within_ties(got, o["indicator"][g], n_k)
                k_rows = inp["k"][l][b, g].float().cpu().numpy()
                v_rows = inp["v"][l][b, g].float().cpu().numpy()
                np.testing.assert_array_equal(res.k_out[l][b, g, : n_k + S_w].float().cpu().numpy(),
                                              co.compact(k_rows, got, S_w))
                np.testing.assert_array_equal(res.v_out[l][b, g, : n_k + S_w].float().cpu().numpy(),
                                              co.compact(v_rows, got, S_w))
                np.testing.assert_array_equal(res.ind_out[l][b, g, :n_k].cpu().numpy(),
                                              res.indicator[l][b, g].cpu().numpy()[got])
    say(f"  positions differing from the oracle's own selection (ties at the cut): {swaps}")
    return res, inp


def test_pass_tiny(cake):
    say("pass tiny")
    res, inp = _check_pass(cake, CONFIGS[1])
    assert res.budgets.sum() == CONFIGS[1].total_budget


def test_pass_bf16_llama_shape_reduced(cake):
    say("pass bf16 reduced")
    cfg = CONFIGS[2].scaled(n_layers=4, seq_len=4096 + 32 + 11, total_budget=4 * 640)
    _check_pass(cake, cfg)


def test_pass_batch_has_per_sequence_budgets(cake):
    say("pass batch")
    cfg = CONFIGS[5].scaled(n_layers=3, batch=2, seq_len=1536, total_budget=3 * 256)
    res, _ = _check_pass(cake, cfg)
    assert res.budgets.shape == (3, 2)


@pytest.mark.parametrize("mode", [1, 2, 3, 4])
def test_pass_indicator_ablation_modes(cake, mode):
    # Mean, Var and Mean*Var in place of Mean + gamma*Var (the paper's indicator ablation), and the
    # accumulated attention of the window rows (Sec. 5.5)
    say(f"pass indicator mode {mode}")
    cfg = CONFIGS[2].scaled(n_layers=2, seq_len=2048 + 32 + 19, total_budget=2 * 400)
    _check_pass(cake, cfg, cake.make_params(indicator_mode=mode))
    cfg = CONFIGS[4].scaled(n_layers=1, seq_len=1500, total_budget=300)
    _check_pass(cake, cfg, cake.make_params(indicator_mode=mode, pool_kernel=1))


def test_pass_is_deterministic(cake):
    say("pass determinism")
    cfg = CONFIGS[2].scaled(n_layers=2, seq_len=3000, total_budget=2 * 300)
    inp = make_config_inputs(cfg, device=DEV)
    q = [inp["q_win"][l] for l in range(2)]
    k = [inp["k"][l] for l in range(2)]
    v = [inp["v"][l] for l in range(2)]
    ev = cake.EvictionPass(q, k, v, cfg.total_budget)
    r1 = ev.run()
    torch.cuda.synchronize()
    ind1 = ev.indicator.clone(); pref1 = r1.pref.copy(); idx1 = [t.clone() for t in r1.idx]
    r2 = ev.run()
    torch.cuda.synchronize()
    assert torch.equal(ind1, ev.indicator) and np.array_equal(pref1, r2.pref)
    assert all(torch.equal(a, b) for a, b in zip(idx1, r2.idx))
