"""CPU fp64 oracle for the CAKE prefill eviction pass.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the HIP library must compute.  It
is imported only by the tests, by the smoke check and by the benchmark's CPU
baseline leg; the product path never calls it and shares no code with it.

Every function follows a passage of the paper (CAKE: cascading and adaptive
KV-cache eviction with layer preferences) and says which.  Arrays are NumPy
float64; inputs in bf16/fp32 are upcast by the caller, so the oracle sees the
same rounded values as the GPU.  Matmul and sort are library primitives; there is
no blocking, fusion or reordering beyond what the definitions state.

Readings taken where the paper is silent (each also listed in the design notes):
  * softmax normalises over every causally visible key (prefix and window) and
    the prefix columns are sliced afterwards, as in Eq. (6)'s A[-S_w:, :-S_w];
  * entropy uses the natural log on the un-renormalised sub-rows, summed over rows;
  * Var is the unbiased estimator by default (`var_correction = 1`);
  * head statistics are averaged over query heads before the powers of Eq. (6);
  * under GQA each query head's Mean + gamma*Var is formed first and the G heads
    of a KV group are then averaged;
  * the pooling layer of Sec. 4.3 is a stride-1 max-pool of odd width over the
    prefix positions with clipped edges, applied after the group average;
  * B_l counts the window tokens (Eq. 11 gives them the score Omega), so
    k_l = B_l - S_w prefix tokens are selected;
  * real-valued budgets of Eq. (7)/(9) become integers by Webster (Sainte-Lague)
    divisor apportionment with a floor of S_w and a cap of N per layer;
  * top-k breaks ties towards the lower position and returns ascending positions;
  * in the decoding phase the pooled attention row of the new token is added to the stored
    indicator (the paper names `update_score` without defining it) and the row that leaves the
    window starts from 0;
  * the quantised form of the retained cache (appendix on compatibility with quantisation
    methods, which combines the method with a 4-bit key-per-channel / value-per-token
    quantiser) is asymmetric uniform b-bit quantisation over groups of 32: keys per channel
    over 32 consecutive retained tokens, values per token over 32 consecutive channels; the
    window rows stay as they are.  Scales and codes are formed in float32, the precision in
    which the library decides them (a code is an integer decided by floating point).

Pins (tests/test_oracle_pins.py): a hand-derived rational worked example,
closed forms for uniform attention, zero temporal variance under static
attention, library softmax / variance / max-pool / sort on special cases,
brute-force apportionment and top-k, Proposition 1 and Theorem 2; for the quantiser
exact reproduction of values on the grid, the half-step error bound, a brute-force
nearest-level search and the key/value group orientation.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class OracleParams:
    scale: Optional[float] = None   # None -> 1/sqrt(head_dim)   (Sec. 2, attention weights)
    gamma: float = 200.0            # App. "More implementation details"
    tau1: float = 1.0               # Eq. (6)
    tau2: float = 1.0
    var_correction: int = 1
    pool_kernel: int = 7
    indicator_mode: int = 0         # 0 Mean + gamma*Var (Eq. 11); 1 Mean; 2 Var; 3 Mean*Var (indicator ablation);
                                    # 4 accumulated attention of the window rows (Sec. 5.5, H2O-style indicator)


# ----------------------------------------------------------------------------------------
# Observation-window attention (Sec. 2 attention weights; Sec. 4.1 recent-window submatrix)
# ----------------------------------------------------------------------------------------
def window_logits(q_win: np.ndarray, k: np.ndarray, scale: Optional[float] = None) -> np.ndarray:
    """s[h, r, j] = scale * <Q_w[h, r], K[h // G, j]>, masked to -inf where key j lies after
    the query (window row r sits at absolute position N - S_w + r).  q_win [H_q,S_w,d], k [H_kv,N,d]."""
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    h_q, s_w, d = q_win.shape
    h_kv, n, _ = k.shape
    group = h_q // h_kv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    s = np.empty((h_q, s_w, n), dtype=np.float64)
    for h in range(h_q):
        s[h] = (q_win[h] @ k[h // group].T) * scale
    query_pos = (n - s_w) + np.arange(s_w)
    key_pos = np.arange(n)
    hidden = key_pos[None, :] > query_pos[:, None]
    s[:, hidden] = -np.inf
    return s


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Row softmax over the last axis (Sec. 2: A = Softmax(Q K^T / sqrt(D)))."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def window_attention(q_win, k, scale=None) -> np.ndarray:
    """A[h, r, :] for the last S_w queries over all N keys."""
    return softmax_rows(window_logits(q_win, k, scale))


def window_attention_given_lse(q_win, k, row_lse: np.ndarray, scale=None) -> np.ndarray:
    """A[h, r, j] = exp(s[h, r, j] - lse[h, r]) with the rows' log-sum-exp supplied by the caller
    (natural log), the form the softmax of Sec. 2 takes once its denominator is known; hidden keys
    get weight 0.  Equals window_attention when lse[h, r] = ln sum_j exp(s[h, r, j])."""
    s = window_logits(q_win, k, scale)
    return np.exp(s - np.asarray(row_lse, dtype=np.float64)[..., None])


def observed(a: np.ndarray, window: int) -> np.ndarray:
    """A[-S_w:, :-S_w] of Eq. (6): the window queries' weights on the prefix keys."""
    return a[..., : a.shape[-1] - window]


# ----------------------------------------------------------------------------------------
# Attention dynamics (Sec. 3) and layer preference (Sec. 4.1)
# ----------------------------------------------------------------------------------------
def dispersion(a_obs: np.ndarray) -> np.ndarray:
    """Eq. (4): H = -sum_i A[i,:] . log(A[i,:])^T per head (0 log 0 taken as 0).  [H_q]"""
    with np.errstate(divide="ignore", invalid="ignore"):
        term = np.where(a_obs > 0.0, a_obs * np.log(a_obs), 0.0)
    return -np.sum(term, axis=(-2, -1))


def column_variance(a_obs: np.ndarray, var_correction: int = 1) -> np.ndarray:
    """Var(A[:, j]) over the S_w window rows, per head and prefix column."""
    s_w = a_obs.shape[-2]
    mu = np.sum(a_obs, axis=-2, keepdims=True) / s_w
    return np.sum((a_obs - mu) ** 2, axis=-2) / (s_w - var_correction)


def shift(a_obs: np.ndarray, var_correction: int = 1) -> np.ndarray:
    """Eq. (5): V = sum_j Var(A[:, j]) per head.  [H_q]"""
    return np.sum(column_variance(a_obs, var_correction), axis=-1)


def layer_preference(h_heads: np.ndarray, v_heads: np.ndarray, tau1: float = 1.0, tau2: float = 1.0
                     ) -> Tuple[float, float, float]:
    """Eq. (6): P = H^(1/tau1) * V^(1/tau2), with the heads of the layer averaged first."""
    h_layer = float(np.mean(h_heads))
    v_layer = float(np.mean(v_heads))
    return h_layer ** (1.0 / tau1) * v_layer ** (1.0 / tau2), h_layer, v_layer


# ----------------------------------------------------------------------------------------
# Attention-shift tolerant eviction indicator (Sec. 4.3)
# ----------------------------------------------------------------------------------------
def head_indicator(a_obs: np.ndarray, gamma: float, var_correction: int = 1, mode: int = 0) -> np.ndarray:
    """Eq. (11), prefix case: Mean(A[-S_w:, n]) + gamma * Var(A[-S_w:, n]).  [H_q, N_p]
    Modes 1-3 are the alternatives of the paper's indicator ablation: Mean, Var, Mean * Var.
    Mode 4 is the accumulated-attention indicator of Sec. 5.5's compatibility experiment taken
    over the observation window: the column sum of the S_w window rows."""
    s_w = a_obs.shape[-2]
    mean = np.sum(a_obs, axis=-2) / s_w
    var = column_variance(a_obs, var_correction)
    if mode == 0:
        return mean + gamma * var
    if mode == 1:
        return mean
    if mode == 2:
        return var
    if mode == 3:
        return mean * var
    if mode == 4:
        return np.sum(a_obs, axis=-2)
    raise ValueError("indicator mode")


def group_reduce(i_q: np.ndarray, group: int) -> np.ndarray:
    """Query-head indicators -> KV-head indicators: mean over each group's G heads."""
    h_q, n_p = i_q.shape
    return i_q.reshape(h_q // group, group, n_p).sum(axis=1) / group


def max_pool(x: np.ndarray, width: int) -> np.ndarray:
    """Stride-1 max over [j - width//2, j + width//2] clipped to the row (Sec. 4.3 pooling layer)."""
    if width == 1:
        return x.copy()
    half = width // 2
    n = x.shape[-1]
    out = np.empty_like(x)
    for j in range(n):
        lo, hi = max(0, j - half), min(n, j + half + 1)
        out[..., j] = np.max(x[..., lo:hi], axis=-1)
    return out


def eviction_indicator(a_obs: np.ndarray, group: int, p: OracleParams) -> np.ndarray:
    """I[g, n] for prefix positions n < N - S_w.  The window positions carry Omega in
    Eq. (11): they are always retained and are not part of this array."""
    i_q = head_indicator(a_obs, p.gamma, p.var_correction, p.indicator_mode)
    return max_pool(group_reduce(i_q, group), p.pool_kernel)


def layer_pass(q_win, k, p: OracleParams, row_lse: Optional[np.ndarray] = None) -> dict:
    """Everything one layer contributes before allocation: indicator [H_kv,N_p], H_h, V_h, P.
    With row_lse [H_q, S_w] the rows are normalised by the supplied log-sum-exp instead."""
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    h_q, s_w, _ = q_win.shape
    h_kv, n, _ = k.shape
    group = h_q // h_kv
    ind = np.empty((h_kv, n - s_w), dtype=np.float64)
    h_heads = np.empty(h_q)
    v_heads = np.empty(h_q)
    for g in range(h_kv):                       # one KV group at a time only to bound memory
        heads = slice(g * group, (g + 1) * group)
        if row_lse is None:
            a_full = window_attention(q_win[heads], k[g: g + 1], p.scale)
        else:
            a_full = window_attention_given_lse(q_win[heads], k[g: g + 1], np.asarray(row_lse)[heads], p.scale)
        a_obs = observed(a_full, s_w)
        h_heads[heads] = dispersion(a_obs)
        v_heads[heads] = shift(a_obs, p.var_correction)
        ind[g] = eviction_indicator(a_obs, group, p)[0]
    pref, h_layer, v_layer = layer_preference(h_heads, v_heads, p.tau1, p.tau2)
    return {"indicator": ind, "h_heads": h_heads, "v_heads": v_heads, "H": h_layer, "V": v_layer, "pref": pref}


# ----------------------------------------------------------------------------------------
# Preference-prioritised allocation, cascading form (Sec. 4.1 Eq. 7, Sec. 4.2 Eq. 9)
# ----------------------------------------------------------------------------------------
def cascade_allocate(pref: Sequence[float], total_budget: int, window: int, seq_len: int) -> List[int]:
    """Integer budgets B_l^(m) for the m+1 = len(pref) layers seen so far.

    Eq. (9) asks for B_l = P_l / sum_k P_k * B_total.  Integers with the exact sum come from
    divisor apportionment: every layer first holds its S_w window tokens, then the remaining
    tokens are awarded one at a time to the layer with the largest P_l / (B_l + 1/2) among
    layers still below N, ties to the lower layer.  If all layers fit whole nothing is evicted.
    """
    pref = [float(x) for x in pref]
    m1 = len(pref)
    if m1 == 0:
        return []
    if any((not math.isfinite(x)) or x < 0.0 for x in pref):
        raise ValueError("preferences must be finite and non-negative")
    if total_budget < m1 * window:
        raise ValueError("total budget smaller than the layers' windows")
    if m1 * seq_len <= total_budget:
        return [seq_len] * m1
    if all(x == 0.0 for x in pref):
        pref = [1.0] * m1
    budgets = [window] * m1
    remaining = total_budget - m1 * window
    prio = np.array([pref[l] / (budgets[l] + 0.5) if budgets[l] < seq_len else -1.0 for l in range(m1)])
    while remaining > 0:
        l = int(np.argmax(prio))                # first maximum: ties go to the lower layer
        if prio[l] < 0.0:
            break
        budgets[l] += 1
        remaining -= 1
        prio[l] = pref[l] / (budgets[l] + 0.5) if budgets[l] < seq_len else -1.0
    return budgets


# ----------------------------------------------------------------------------------------
# EVICT (Sec. 4.3 Eq. 12): top-k positions, compaction
# ----------------------------------------------------------------------------------------
def select_topk(indicator_row: np.ndarray, k: int) -> np.ndarray:
    """Positions of the k largest entries under (value descending, position ascending),
    returned in ascending position order."""
    x = np.asarray(indicator_row)
    order = np.argsort(-x, kind="stable")       # stable: equal values keep position order
    return np.sort(order[:k]).astype(np.int64)


def compact(rows: np.ndarray, idx: np.ndarray, window: int) -> np.ndarray:
    """K_hat = K[D, :] with the S_w window rows (the tail of `rows`) kept after them."""
    return np.concatenate([rows[idx], rows[rows.shape[0] - window:]], axis=0)


def evict(k_rows: np.ndarray, v_rows: np.ndarray, indicator_row: np.ndarray, budget: int, window: int):
    """EVICT({K,V}, B, I) of Alg. 1 for one head.  k_rows/v_rows [cur+S_w, d]; indicator_row [cur].
    Returns (K_hat, V_hat, I_hat, idx) with idx relative to the current (possibly compacted) rows."""
    cur = indicator_row.shape[0]
    keep = min(max(budget - window, 0), cur)
    idx = select_topk(indicator_row, keep)
    return compact(k_rows, idx, window), compact(v_rows, idx, window), indicator_row[idx], idx


# ----------------------------------------------------------------------------------------
# Whole pass: one-shot (Sec. 4.1) and cascading (Sec. 4.2, Alg. 1)
# ----------------------------------------------------------------------------------------
def one_shot(prefs, indicators, ks, vs, total_budget: int, window: int):
    """Eq. (7) budgets from all layers' preferences, then EVICT once per layer and head.
    indicators[l] [H_kv,N_p]; ks[l], vs[l] [H_kv,N,d].  Returns budgets and per-layer results."""
    n = ks[0].shape[1]
    budgets = cascade_allocate(prefs, total_budget, window, n)
    out = []
    for l, b_l in enumerate(budgets):
        heads = [evict(ks[l][g], vs[l][g], indicators[l][g], b_l, window) for g in range(ks[l].shape[0])]
        out.append({"k": [h[0] for h in heads], "v": [h[1] for h in heads],
                    "ind": [h[2] for h in heads], "pos": [h[3] for h in heads]})
    return budgets, out


def cascade_manage(prefs, indicators, ks, vs, total_budget: int, window: int):
    """Alg. 1.  Stage m admits layer m, recomputes B^(m) over layers 0..m (Eq. 9) and applies EVICT
    to every admitted layer's current cache and indicator.  `pos` maps retained rows back to the
    original prefix positions.  Returns the per-stage budgets and the final caches."""
    n_layers = len(prefs)
    n = ks[0].shape[1]
    cache: List[dict] = []
    history: List[List[int]] = []
    for m in range(n_layers):
        h_kv = ks[m].shape[0]
        cache.append({"k": [ks[m][g] for g in range(h_kv)], "v": [vs[m][g] for g in range(h_kv)],
                      "ind": [indicators[m][g] for g in range(h_kv)],
                      "pos": [np.arange(n - window, dtype=np.int64) for _ in range(h_kv)]})
        budgets = cascade_allocate(prefs[: m + 1], total_budget, window, n)
        history.append(budgets)
        for l in range(m + 1):
            c = cache[l]
            for g in range(len(c["k"])):
                k_hat, v_hat, i_hat, idx = evict(c["k"][g], c["v"][g], c["ind"][g], budgets[l], window)
                c["k"][g], c["v"][g], c["ind"][g], c["pos"][g] = k_hat, v_hat, i_hat, c["pos"][g][idx]
    return history, cache


# ----------------------------------------------------------------------------------------
# Decode-phase maintenance (implementation appendix, decoding branch of the listing)
# ----------------------------------------------------------------------------------------
def decode_update(q_new: np.ndarray, k_rows: np.ndarray, indicator: np.ndarray, window: int, p: OracleParams
                  ) -> np.ndarray:
    """One generated token: q_new [H_q, d] attends to all cached rows k_rows [H_kv, n, d] (the last
    `window` of them are the window, the newest row last); softmax over all n rows per head; the
    weights on the n - window scored rows are averaged over each KV group, max-pooled, and ADDED to
    the stored indicator [H_kv, n - window].  Reading: the paper names the update (`update_score`)
    without defining it; a single query row has a mean but no variance, so gamma plays no part."""
    q_new = np.asarray(q_new, dtype=np.float64)
    k_rows = np.asarray(k_rows, dtype=np.float64)
    h_q, d = q_new.shape
    h_kv, n, _ = k_rows.shape
    group = h_q // h_kv
    scale = p.scale if p.scale is not None else 1.0 / math.sqrt(d)
    s = np.empty((h_q, n))
    for h in range(h_q):
        s[h] = (k_rows[h // group] @ q_new[h]) * scale
    a = softmax_rows(s)                                  # the new token sees every cached row
    obs = a[:, : n - window]
    per_kv = obs.reshape(h_kv, group, n - window).sum(axis=1) / group
    return np.asarray(indicator, dtype=np.float64) + max_pool(per_kv, p.pool_kernel)


def decode_step(q_new, cache: dict, k_new, v_new, window: int, p: OracleParams) -> dict:
    """Append the new token, update the indicator (decode_update) and evict one scored row per
    head so that the cache returns to its size (EVICT at k = cur, Eq. 12).  cache = {"k", "v":
    [H_kv, cur + window, d], "ind": [H_kv, cur]}; the row that leaves the window enters the scored
    part with indicator 0."""
    k = np.concatenate([cache["k"], np.asarray(k_new, dtype=np.float64)[:, None, :]], axis=1)
    v = np.concatenate([cache["v"], np.asarray(v_new, dtype=np.float64)[:, None, :]], axis=1)
    h_kv, cur = cache["ind"].shape
    ind = np.concatenate([cache["ind"], np.zeros((h_kv, 1))], axis=1)
    ind = decode_update(q_new, k, ind, window, p)
    out = {"k": [], "v": [], "ind": [], "idx": []}
    for g in range(h_kv):
        sel = select_topk(ind[g], cur)
        out["idx"].append(sel)
        out["k"].append(compact(k[g], sel, window))
        out["v"].append(compact(v[g], sel, window))
        out["ind"].append(ind[g][sel])
    return {"k": np.stack(out["k"]), "v": np.stack(out["v"]), "ind": np.stack(out["ind"]), "idx": np.stack(out["idx"])}


# ----------------------------------------------------------------------------------------
# Quantised storage of the retained cache (appendix "Comparison and compatibility with
# quantization methods": eviction combined with key-per-channel / value-per-token quantisation)
# ----------------------------------------------------------------------------------------
QUANT_GROUP = 32


def quantize_uniform(x: np.ndarray, bits: int, axis: int, group: int = QUANT_GROUP):
    """Asymmetric uniform quantisation to `bits` bits over groups of `group` consecutive entries
    along `axis` (the last group may be shorter): zero = group minimum, scale = (max - min) /
    (2^bits - 1), code = round-half-even((x - zero) / scale) in [0, 2^bits - 1]; a constant group
    has scale 0 and codes 0.  float32 throughout.  Returns (codes uint8 like x, scale, zero) with
    the group index in place of `axis`."""
    x = np.moveaxis(np.asarray(x, dtype=np.float32), axis, -1)
    levels = np.float32(2 ** bits - 1)
    n = x.shape[-1]
    n_groups = -(-n // group)
    codes = np.zeros(x.shape, dtype=np.uint8)
    scale = np.zeros(x.shape[:-1] + (n_groups,), dtype=np.float32)
    zero = np.zeros_like(scale)
    for gi in range(n_groups):
        seg = x[..., gi * group:(gi + 1) * group]
        lo, hi = seg.min(axis=-1), seg.max(axis=-1)
        sc = ((hi - lo) / levels).astype(np.float32)
        with np.errstate(divide="ignore", invalid="ignore"):
            c = np.rint(((seg - lo[..., None]).astype(np.float32) / sc[..., None]).astype(np.float32))
        c = np.where(sc[..., None] > 0, np.clip(c, 0, levels), 0)
        codes[..., gi * group:(gi + 1) * group] = c.astype(np.uint8)
        scale[..., gi], zero[..., gi] = sc, lo
    return np.moveaxis(codes, -1, axis), np.moveaxis(scale, -1, axis), np.moveaxis(zero, -1, axis)


def dequantize_uniform(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray, axis: int, group: int = QUANT_GROUP):
    """x ~ zero + code * scale with each group's scale and zero spread over its entries."""
    n = codes.shape[axis]
    rep = lambda a: np.repeat(a, group, axis=axis).take(np.arange(n), axis=axis)
    return rep(zero).astype(np.float64) + codes.astype(np.float64) * rep(scale).astype(np.float64)


def quantize_cache(k_rows: np.ndarray, v_rows: np.ndarray, bits: int):
    """The retained prefix rows of one head, k_rows / v_rows [keep, d]: keys per channel over
    groups of 32 tokens (scale, zero [ceil(keep/32), d]), values per token over groups of 32
    channels (scale, zero [keep, d/32])."""
    return quantize_uniform(k_rows, bits, axis=0), quantize_uniform(v_rows, bits, axis=1)
