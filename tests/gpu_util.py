"""Helpers shared by the GPU parity tests: build the library if needed, run the oracle on
host copies of the very tensors the GPU saw, and compare to the stated bars."""
import os
import sys

import numpy as np
import torch

from oracle import cake_oracle as co

RTOL = 1e-3      # indicators, H, V, P: relative error bar on bf16/fp32 inputs
ATOL = 1e-30     # entries that underflow in fp32


def load_cake():
    import paper_2503_12491_amd as pkg
    from paper_2503_12491_amd import _ffi
    if not os.path.exists(_ffi.LIB_PATH):
        from paper_2503_12491_amd.build import build
        build()
    return pkg


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def oracle_params(params) -> co.OracleParams:
    return co.OracleParams(scale=(params.scale if params.scale > 0 else None), gamma=params.gamma, tau1=params.tau1,
                           tau2=params.tau2, var_correction=params.var_correction, pool_kernel=params.pool_kernel,
                           indicator_mode=params.indicator_mode)


def host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_layer(q_win_b, k_b, params, row_lse_b=None):
    """Oracle pass for one (layer, sequence): q_win_b [H_q,S_w,d], k_b [H_kv,N,d] device tensors
    (and, for the hand-off path, the same f32 row normalisers [H_q,S_w] the GPU was given)."""
    return co.layer_pass(host64(q_win_b), host64(k_b), oracle_params(params),
                         None if row_lse_b is None else host64(row_lse_b))


def oracle_slice(q_win_b, k_b, g, group, params):
    """Oracle indicator of ONE KV head g (plus its heads' H_h, V_h) for a (layer, sequence)."""
    p = oracle_params(params)
    q = host64(q_win_b[g * group:(g + 1) * group])
    k = host64(k_b[g:g + 1])
    s_w = q.shape[1]
    a_obs = co.observed(co.window_attention(q, k, p.scale), s_w)
    return {"indicator": co.eviction_indicator(a_obs, group, p)[0], "h_heads": co.dispersion(a_obs),
            "v_heads": co.shift(a_obs, p.var_correction)}


def assert_close(got, want, what, rtol=RTOL, atol=ATOL):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want) / np.maximum(np.abs(want), atol / rtol)
    worst = float(err.max()) if err.size else 0.0
    assert worst <= rtol, f"{what}: max relative error {worst:.3e} > {rtol}"
    return worst


def assert_topk_within_ties(got_idx, oracle_ind_row, k, rtol=RTOL):
    """End-to-end selection check against the oracle's own indicator: the two index sets may
    differ only at positions whose oracle indicator is within rtol of the k-th largest value."""
    want = co.select_topk(oracle_ind_row, k)
    got = np.asarray(got_idx, dtype=np.int64)
    assert got.shape == want.shape and np.all(np.diff(got) > 0)
    if k == 0 or k == oracle_ind_row.shape[0]:
        np.testing.assert_array_equal(got, want)
        return 0
    kth = np.sort(oracle_ind_row)[::-1][k - 1]
    diff = np.setxor1d(got, want)
    if diff.size:
        vals = oracle_ind_row[diff]
        # each of the two indicators is within rtol of the oracle's, so two entries can change
        # places only when they lie within 2*rtol of each other, i.e. of the k-th value
        assert np.all(np.abs(vals - kth) <= 2 * rtol * abs(kth)), "selection differs away from the k-th cut"
    return int(diff.size)


def torch_row_lse(q_win_l: torch.Tensor, k_l: torch.Tensor, scale=None) -> torch.Tensor:
    """Stand-in for what a prefill attention kernel hands over: ln sum_j exp(scale*<q_r,k_j>) over the
    keys visible to each window row, computed by torch in fp64 and rounded to f32.  [B, H_q, S_w]."""
    B, H_q, S_w, d = q_win_l.shape
    H_kv, N = k_l.shape[1], k_l.shape[2]
    G = H_q // H_kv
    scale = scale if scale else d ** -0.5
    q = q_win_l.double().view(B, H_kv, G, S_w, d)
    s = torch.einsum("bgwrd,bgnd->bgwrn", q, k_l.double()) * scale
    pos_q = (N - S_w) + torch.arange(S_w, device=s.device)
    hidden = torch.arange(N, device=s.device)[None, :] > pos_q[:, None]
    s = s.masked_fill(hidden, float("-inf"))
    return torch.logsumexp(s, dim=-1).view(B, H_q, S_w).float().contiguous()
