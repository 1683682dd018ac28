"""Stage driver for the eviction pass: sequences the five libcake calls (Alg. 1 / Sec. 4.1).

Orchestration and buffer management only; every computation happens inside libcake.
One-shot mode (Sec. 4.1): scores for all layers, Eq. 7 budgets and the placement of the outputs on
the device (cake_plan_eviction), top-k and compaction for all layers (cake_evict_planned); the host
reads the plan back once at the end.  Cascade mode (Sec. 4.2, Alg. 1): stage m admits layer
m, recomputes B^(m) and re-evicts layers 0..m from their already compacted caches.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as C


@dataclass
class PassResult:
    budgets: np.ndarray                 # [L, B] int, window tokens included
    keep: np.ndarray                    # [L, B] prefix tokens retained
    pref: np.ndarray                    # [B, L] float64
    hv: np.ndarray                      # [B, L, 2] float64 (H_l, V_l)
    indicator: List[torch.Tensor]       # per layer [B, H_kv, N_p] f32 (pooled)
    idx: List[torch.Tensor]             # per layer [B, H_kv, cap_l] int32 ascending positions
    k_out: List[torch.Tensor]           # per layer [B, H_kv, cap_l + S_w, d]
    v_out: List[torch.Tensor]
    ind_out: List[torch.Tensor]         # per layer [B, H_kv, cap_l] f32
    stage_budgets: list = field(default_factory=list)   # cascade mode: budgets after every stage


def _strides3(t: torch.Tensor):
    assert t.dim() == 4 and t.stride(3) == 1, "expect [B, H, rows, d] with contiguous d"
    return [t.stride(0), t.stride(1), t.stride(2)]


class EvictionPass:
    """Buffers and call sequence for one prompt's eviction pass on one GPU."""

    def __init__(self, q_win: Sequence[torch.Tensor], k: Sequence[torch.Tensor], v: Sequence[torch.Tensor],
                 total_budget: int, params=None, row_lse: Optional[Sequence[torch.Tensor]] = None):
        """row_lse: per layer [B, H_q, S_w] f32 log-sum-exp of the window rows, if the prefill attention
        already produced it; the scores then take one pass over K (cake_window_scores_lse)."""
        self.q_win, self.k, self.v = list(q_win), list(k), list(v)
        q0, k0 = self.q_win[0], self.k[0]
        self.L = len(self.k)
        self.B, self.H_q, self.S_w, self.d = q0.shape
        self.H_kv, self.N = k0.shape[1], k0.shape[2]
        self.N_p = self.N - self.S_w
        self.total_budget = int(total_budget)
        self.dev = k0.device
        self.dtype = k0.dtype
        self.params = params if params is not None else C.make_params()
        self.shape = C.make_shape(self.B, self.L, self.H_q, self.H_kv, self.d, self.N, self.S_w, self.dtype)
        for t in self.q_win[1:]:
            assert _strides3(t) == _strides3(q0)
        for t in self.k[1:] + self.v:
            assert _strides3(t) == _strides3(k0)

        self.workspace = torch.empty(C.cake_workspace_bytes(self.shape), dtype=torch.uint8, device=self.dev)
        self.indicator = torch.empty(self.L, self.B, self.H_kv, self.N_p, dtype=torch.float32, device=self.dev)
        self.pref = torch.empty(self.B, self.L, dtype=torch.float64, device=self.dev)
        self.hv = torch.empty(self.B, self.L, 2, dtype=torch.float64, device=self.dev)
        self.pref_host = torch.empty(self.B, self.L, dtype=torch.float64).pin_memory()
        self.hv_host = torch.empty(self.B, self.L, 2, dtype=torch.float64).pin_memory()

        self.tbl_q = C.ptr_table(self.q_win)
        self.tbl_k = C.ptr_table(self.k)
        self.tbl_v = C.ptr_table(self.v)
        self.tbl_ind = C.ptr_table([self.indicator[l] for l in range(self.L)])
        self.row_lse = None if row_lse is None else [t.contiguous() for t in row_lse]
        if self.row_lse is not None:
            for t in self.row_lse:
                assert t.dtype == torch.float32 and tuple(t.shape) == (self.B, self.H_q, self.S_w)
            self.tbl_lse = C.ptr_table(self.row_lse)

        # Output pools.  Row capacity of layer l is cap_l = max_b keep[l, b]; over all layers
        # sum_l cap_l <= B * (B_total - L*S_w), and exactly B_total - L*S_w when B = 1.
        max_rows = min(self.B * max(self.total_budget - self.L * self.S_w, 0), self.L * self.N_p)
        rows_kv = max_rows + self.L * self.S_w
        bh = self.B * self.H_kv
        self.pool_k = torch.empty(bh * rows_kv * self.d, dtype=self.dtype, device=self.dev)
        self.pool_v = torch.empty_like(self.pool_k)
        self.pool_idx = torch.empty(bh * max(max_rows, 1), dtype=torch.int32, device=self.dev)
        self.pool_ind = torch.empty(bh * max(max_rows, 1), dtype=torch.float32, device=self.dev)
        self._cur_full = [self.N_p] * (self.L * self.B)
        self._strides_full = [_strides3(k0)] * self.L
        self.tbl_out_host = torch.empty(4, self.L, dtype=torch.int64).pin_memory()
        self.tbl_out = torch.empty(4, self.L, dtype=torch.int64, device=self.dev)
        # device-resident plan of the one-shot pass (budgets, keep counts, output places) and its host copy
        self.plan = torch.empty(C.cake_plan_bytes(self.shape), dtype=torch.uint8, device=self.dev)
        self.plan_host = torch.empty(self.plan.numel(), dtype=torch.uint8).pin_memory()
        self.status = torch.empty(self.B, dtype=torch.int32, device=self.dev)
        self.status_host = torch.empty(self.B, dtype=torch.int32).pin_memory()

    # ------------------------------------------------------------------ the five calls
    def scores(self, stream=None) -> None:
        if self.row_lse is None:
            C.cake_window_scores(self.shape, self.params, self.tbl_q, self.tbl_k, _strides3(self.q_win[0]),
                                 _strides3(self.k[0]), self.tbl_ind, self.workspace, stream)
        else:
            C.cake_window_scores_lse(self.shape, self.params, self.tbl_q, self.tbl_k, _strides3(self.q_win[0]),
                                     _strides3(self.k[0]), self.tbl_lse, self.tbl_ind, self.workspace, stream)
        C.cake_layer_preference(self.shape, self.params, self.workspace, self.pref, self.hv, stream)

    def scores_segmented(self, segment_keys: int, fetch=None, stream=None) -> None:
        """The score stage with the keys handed over `segment_keys` positions at a time (a
        multiple of cake_scores_chunk_keys), as a caller would whose K is not resident: both
        passes walk the segments, every segment copied into a staging buffer of that size first.
        `fetch(l, lo, hi)` returns layer l's keys [B, H_kv, hi - lo, d]; the default slices self.k.
        Bit-identical to scores()."""
        chunk = C.cake_scores_chunk_keys(self.shape)
        assert segment_keys > 0 and segment_keys % chunk == 0, f"segment of {segment_keys} keys is not a multiple of {chunk}"
        fetch = fetch or (lambda l, lo, hi: self.k[l][:, :, lo:hi])
        stage = [torch.empty(self.B, self.H_kv, min(segment_keys, self.N), self.d, dtype=self.dtype, device=self.dev)
                 for _ in range(self.L)]
        tbl = C.ptr_table(stage)
        qs, ks = _strides3(self.q_win[0]), _strides3(stage[0])
        for which, end in ((1, self.N), (2, self.N_p)):
            for lo in range(0, end, segment_keys):
                hi = min(lo + segment_keys, self.N)
                for l in range(self.L):
                    stage[l][:, :, : hi - lo].copy_(fetch(l, lo, hi))
                    if hi - lo < stage[l].shape[2]:
                        stage[l][:, :, hi - lo:].fill_(float("nan"))      # must never be read
                C.cake_window_scores_segment(self.shape, self.params, which, lo, hi - lo, self.tbl_q, tbl, qs, ks,
                                             self.workspace, stream)
            C.cake_window_scores_finish(self.shape, self.params, which, self.tbl_ind if which == 2 else None,
                                        self.workspace, stream)
        C.cake_layer_preference(self.shape, self.params, self.workspace, self.pref, self.hv, stream)

    def preferences_to_host(self):
        """The pass's one device-to-host crossing: L*B preferences (and H, V)."""
        self.pref_host.copy_(self.pref, non_blocking=True)
        self.hv_host.copy_(self.hv, non_blocking=True)
        torch.cuda.current_stream().synchronize()
        return self.pref_host.numpy().copy(), self.hv_host.numpy().copy()

    def allocate(self, pref: np.ndarray) -> np.ndarray:
        """Eq. 7 per sequence.  Returns budgets [L, B]."""
        out = np.empty((self.L, self.B), dtype=np.int64)
        for b in range(self.B):
            out[:, b] = C.cake_cascade_allocate(pref[b], self.total_budget, self.S_w, self.N)
        return out

    def _carve_outputs(self, keep: np.ndarray):
        """Place every layer's outputs in the pools for the given keep counts [L, B]: fills the
        device pointer table (one asynchronous upload) and returns the per-layer element offsets.
        No tensors are created here; `_views` makes them when a result is inspected."""
        caps = keep.max(axis=1).astype(np.int64)
        bh = self.B * self.H_kv
        n_kv = bh * (caps + self.S_w) * self.d
        n_i = bh * caps
        off_kv = np.concatenate([[0], np.cumsum(n_kv)[:-1]])
        off_i = np.concatenate([[0], np.cumsum(n_i)[:-1]])
        th = self.tbl_out_host.numpy()
        th[0] = self.pool_idx.data_ptr() + off_i * 4
        th[1] = self.pool_k.data_ptr() + off_kv * self.pool_k.element_size()
        th[2] = self.pool_v.data_ptr() + off_kv * self.pool_v.element_size()
        th[3] = self.pool_ind.data_ptr() + off_i * 4
        self.tbl_out.copy_(self.tbl_out_host, non_blocking=True)
        return caps, off_kv, off_i

    def _views(self, caps, off_kv, off_i):
        """Per-layer tensor views of the output pools."""
        bh = self.B * self.H_kv
        idx, k_out, v_out, ind_out = [], [], [], []
        for l in range(self.L):
            cap, okv, oi = int(caps[l]), int(off_kv[l]), int(off_i[l])
            n_kv = bh * (cap + self.S_w) * self.d
            n_i = bh * cap
            k_out.append(self.pool_k[okv: okv + n_kv].view(self.B, self.H_kv, cap + self.S_w, self.d))
            v_out.append(self.pool_v[okv: okv + n_kv].view(self.B, self.H_kv, cap + self.S_w, self.d))
            idx.append(self.pool_idx[oi: oi + n_i].view(self.B, self.H_kv, cap))
            ind_out.append(self.pool_ind[oi: oi + n_i].view(self.B, self.H_kv, cap))
        return idx, k_out, v_out, ind_out

    def evict_launch(self, budgets: np.ndarray, stream=None):
        """Top-k and compaction for all layers; returns (keep, placement) without touching the
        outputs."""
        keep = C.cake_keep_counts(budgets, self.N_p, self.S_w)
        placement = self._carve_outputs(keep)
        kk = keep.reshape(-1).tolist()
        C.cake_select_topk(self.shape, self.tbl_ind, self._cur_full, kk, self.tbl_out[0], None, stream)
        C.cake_compact_kv(self.shape, self.tbl_k, self.tbl_v, self._strides_full, self._cur_full, kk, self.tbl_out[0],
                          self.tbl_ind, self.tbl_out[1], self.tbl_out[2], self.tbl_out[3], stream)
        return keep, placement

    def evict(self, budgets: np.ndarray, stream=None):
        keep, placement = self.evict_launch(budgets, stream)
        return (keep,) + self._views(*placement)

    # ------------------------------------------------------------------ whole pass
    def plan_and_evict(self, stream=None) -> None:
        """Eq. 7 budgets, keep counts and output placement on the device, then top-k and
        compaction of all layers from that plan.  Nothing here waits for the GPU."""
        C.cake_plan_eviction(self.shape, self.pref, self.total_budget, None, self.pool_idx, self.pool_k, self.pool_v,
                             self.pool_ind, self.plan, self.status, stream)
        C.cake_evict_planned(self.shape, self.tbl_ind, self.tbl_k, self.tbl_v, _strides3(self.k[0]), self.plan, stream)

    def read_plan(self):
        """Budgets and keep counts [L, B] of the last planned pass, preferences and (H, V): one
        read-back after the whole pass has been enqueued."""
        self.plan_host.copy_(self.plan, non_blocking=True)
        self.status_host.copy_(self.status, non_blocking=True)
        pref, hv = self.preferences_to_host()           # synchronises the stream
        if int(self.status_host.max()) != 0:
            raise C.CakeError(-1, "a layer preference is NaN, negative or infinite")
        budgets, keep, _, _ = C.plan_fields(self.plan_host, self.L, self.B)
        return budgets, keep, pref, hv

    def _placement(self, keep: np.ndarray):
        """Element offsets of every layer's outputs in the pools (the rule cake_plan_eviction applies)."""
        caps = keep.max(axis=1).astype(np.int64)
        bh = self.B * self.H_kv
        n_kv = bh * (caps + self.S_w) * self.d
        n_i = bh * caps
        return caps, np.concatenate([[0], np.cumsum(n_kv)[:-1]]), np.concatenate([[0], np.cumsum(n_i)[:-1]])

    def run(self) -> PassResult:
        """One-shot pass (Sec. 4.1): all layers scored, Eq. 7 budgets, one EVICT per layer; the host
        waits once, at the end."""
        self.scores()
        self.plan_and_evict()
        budgets, keep, pref, hv = self.read_plan()
        idx, k_out, v_out, ind_out = self._views(*self._placement(keep))
        return PassResult(budgets, keep, pref, hv, [self.indicator[l] for l in range(self.L)], idx, k_out, v_out,
                          ind_out)

    def run_launch_only(self) -> None:
        """The same pass, enqueued only (what a serving loop, and bench.py, time)."""
        self.scores()
        self.plan_and_evict()

    def run_host_allocated(self) -> PassResult:
        """The one-shot pass with the allocation on the host (cake_cascade_allocate): preferences read
        back, budgets computed, counts handed to cake_select_topk / cake_compact_kv as host arrays."""
        self.scores()
        pref, hv = self.preferences_to_host()
        budgets = self.allocate(pref)
        keep, idx, k_out, v_out, ind_out = self.evict(budgets)
        return PassResult(budgets, keep, pref, hv, [self.indicator[l] for l in range(self.L)], idx, k_out, v_out,
                          ind_out)

    def run_cascade(self, track_positions: bool = True) -> PassResult:
        """Cascading pass (Sec. 4.2, Alg. 1) over the layers this object was built with: every layer
        is admitted to a CascadeSession in turn.  The full pooled indicators are kept for inspection."""
        session = CascadeSession(self.L, self.total_budget, self.params, track_positions=track_positions)
        for m in range(self.L):
            session.admit(self.q_win[m], self.k[m], self.v[m], None if self.row_lse is None else self.row_lse[m],
                          indicator_out=self.indicator[m])
        res = session.result()
        res.indicator = [self.indicator[l] for l in range(self.L)]
        return res


class _Held:
    """Where a layer's current cache lives: raw device addresses into the caller's tensors or into a
    slab this session allocated, the element strides of K/V, the row capacity, and the owners that
    keep the memory alive."""
    __slots__ = ("k", "v", "ind", "strides", "cap", "owners", "views")

    def __init__(self, k, v, ind, strides, cap, owners, views):
        self.k, self.v, self.ind, self.strides, self.cap, self.owners, self.views = k, v, ind, strides, cap, owners, views


class CascadeSession:
    """Alg. 1 as the prefill produces its layers: `admit` takes layer m's window queries, keys and
    values when the forward pass reaches it, scores the layer, recomputes B^(m) over the layers seen
    so far (Eq. 9) and applies EVICT to each of them on its current, already compacted cache and
    indicator, all affected layers batched into one top-k and one compaction call.  A layer whose
    budget did not shrink is left as it is (EVICT would keep everything).  The session references
    the caller's K/V of a layer only until that layer's first eviction, so after every stage it
    holds at most B_total rows per head in all (Sec. 4.2: the prefill's peak stays at the budget
    plus the layer being admitted).  With `track_positions` the retained rows' original prefix
    positions are carried along (index bookkeeping with torch.gather, not part of the method).

    Per stage the host does one pinned read-back of the new layer's preference, the allocation,
    one upload of all pointer tables and four slab allocations (the outputs of every affected layer
    are carved from them); nothing else touches the allocator or the copy engine."""

    _ROWS = 10      # pointer tables per stage: q, k, ind (scores); ind_in, idx, k_in, v_in, k_out, v_out, i_out

    def __init__(self, n_layers: int, total_budget: int, params=None, track_positions: bool = True):
        self.L = int(n_layers)
        self.total_budget = int(total_budget)
        self.params = params if params is not None else C.make_params()
        self.track_positions = track_positions
        self.m = 0                                     # layers admitted so far
        self.held: List[_Held] = []
        self.cur_pos: List[Optional[torch.Tensor]] = []
        self.stage_budgets: list = []
        self.budgets = None
        self._geom = None

    def _setup(self, q_win, k):
        B, H_q, S_w, d = q_win.shape
        H_kv, N = k.shape[1], k.shape[2]
        dev = k.device
        self._geom = (B, H_q, H_kv, S_w, d, N, k.dtype, dev)
        self.shape1 = C.make_shape(B, 1, H_q, H_kv, d, N, S_w, k.dtype)
        self.ws1 = torch.empty(C.cake_workspace_bytes(self.shape1), dtype=torch.uint8, device=dev)
        self.pref1 = torch.empty(3 * B, dtype=torch.float64, device=dev)       # P [B], then (H, V) [B, 2]
        self.pref1_host = torch.empty(3 * B, dtype=torch.float64).pin_memory()
        self.pref = np.zeros((B, self.L))
        self.hv = np.zeros((B, self.L, 2))
        self.cur_len = np.zeros((self.L, B), dtype=np.int64)
        # pointer tables: two pinned staging copies (a stage's upload has certainly run by the time
        # the stage after next refills the same copy: every stage waits for its read-back) and one
        # device copy per parity
        self.tbl_host = [torch.zeros(self._ROWS, self.L, dtype=torch.int64).pin_memory() for _ in range(2)]
        self.tbl_dev = [torch.zeros(self._ROWS, self.L, dtype=torch.int64, device=dev) for _ in range(2)]
        self.elem = torch.empty(0, dtype=k.dtype).element_size()

    def rows_held(self) -> int:
        """Cache rows per KV head and sequence that the session holds now (window rows included)."""
        return int(sum(h.cap + self._geom[3] for h in self.held))

    def admit(self, q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, row_lse: Optional[torch.Tensor] = None,
              indicator_out: Optional[torch.Tensor] = None) -> np.ndarray:
        """Stage m = number of layers admitted before this call.  Returns B^(m), shape [m+1, B]."""
        assert self.m < self.L, "every layer has been admitted"
        if self._geom is None:
            self._setup(q_win, k)
        B, H_q, H_kv, S_w, d, N, dtype, dev = self._geom
        assert tuple(q_win.shape) == (B, H_q, S_w, d) and tuple(k.shape) == (B, H_kv, N, d) and v.shape == k.shape
        assert _strides3(v) == _strides3(k)
        N_p, m = N - S_w, self.m
        host, devt = self.tbl_host[m & 1], self.tbl_dev[m & 1]
        th = host.numpy()
        # ---- admit layer m: indicator and preference
        ind = indicator_out if indicator_out is not None else torch.empty(B, H_kv, N_p, dtype=torch.float32, device=dev)
        lse = None if row_lse is None else row_lse.contiguous()
        th[0, 0], th[1, 0], th[2, 0] = q_win.data_ptr(), k.data_ptr(), ind.data_ptr()
        th[3, 0] = 0 if lse is None else lse.data_ptr()
        devt.copy_(host, non_blocking=True)
        if lse is None:
            C.cake_window_scores(self.shape1, self.params, devt[0], devt[1], _strides3(q_win), _strides3(k), devt[2], self.ws1)
        else:
            C.cake_window_scores_lse(self.shape1, self.params, devt[0], devt[1], _strides3(q_win), _strides3(k),
                                     devt[3], devt[2], self.ws1)
        C.cake_layer_preference(self.shape1, self.params, self.ws1, self.pref1[:B], self.pref1[B:])
        self.pref1_host.copy_(self.pref1, non_blocking=True)
        torch.cuda.current_stream().synchronize()
        got = self.pref1_host.numpy()
        self.pref[:, m] = got[:B]
        self.hv[:, m] = got[B:].reshape(B, 2)
        self.held.append(_Held(k.data_ptr(), v.data_ptr(), ind.data_ptr(), _strides3(k), N_p, (k, v, ind, lse),
                               (k, v, ind)))
        self.cur_len[m, :] = N_p
        self.cur_pos.append(torch.arange(N_p, device=dev, dtype=torch.int64).expand(B, H_kv, N_p)
                            if self.track_positions else None)
        self.m = m + 1
        # ---- B^(m) for the layers seen so far
        budgets = np.empty((m + 1, B), dtype=np.int64)
        for b in range(B):
            budgets[:, b] = C.cake_cascade_allocate(self.pref[b, : m + 1], self.total_budget, S_w, N)
        self.budgets = budgets
        self.stage_budgets.append(budgets.copy())
        keep = C.cake_keep_counts(budgets, self.cur_len[: m + 1], S_w)
        layers = np.nonzero((keep < self.cur_len[: m + 1]).any(axis=1))[0].tolist()
        if not layers:
            return budgets
        # ---- EVICT the affected layers in one batched call each; outputs carved from four slabs
        n = len(layers)
        shape_n = C.make_shape(B, n, H_q, H_kv, d, N, S_w, dtype)
        caps = keep[layers].max(axis=1)                                   # row capacity of each output
        caps1 = np.maximum(caps, 1)
        bh = B * H_kv
        off_kv = np.concatenate([[0], np.cumsum((caps + S_w) * (bh * d))])
        off_i = np.concatenate([[0], np.cumsum(caps1 * bh)])
        k_slab = torch.empty(int(off_kv[-1]), dtype=dtype, device=dev)
        v_slab = torch.empty(int(off_kv[-1]), dtype=dtype, device=dev)
        i_slab = torch.empty(int(off_i[-1]), dtype=torch.float32, device=dev)
        # zero-filled: with a ragged batch the entries past a sequence's own count are never
        # written by the library, and the position bookkeeping below gathers through them
        idx_slab = (torch.zeros if self.track_positions and B > 1 else torch.empty)(
            int(off_i[-1]), dtype=torch.int32, device=dev)
        kb, vb, ib, xb = k_slab.data_ptr(), v_slab.data_ptr(), i_slab.data_ptr(), idx_slab.data_ptr()
        strides, cl, kk = [], [], []
        for j, l in enumerate(layers):
            h = self.held[l]
            th[3, j], th[5, j], th[6, j] = h.ind, h.k, h.v
            th[4, j] = xb + int(off_i[j]) * 4
            th[7, j] = kb + int(off_kv[j]) * self.elem
            th[8, j] = vb + int(off_kv[j]) * self.elem
            th[9, j] = ib + int(off_i[j]) * 4
            strides.append(h.strides)
        cl = self.cur_len[layers].reshape(-1).tolist()
        kk = keep[layers].reshape(-1).tolist()
        devt.copy_(host, non_blocking=True)
        C.cake_select_topk(shape_n, devt[3], cl, kk, devt[4])
        C.cake_compact_kv(shape_n, devt[5], devt[6], strides, cl, kk, devt[4], devt[3], devt[7], devt[8], devt[9])
        for j, l in enumerate(layers):
            c, c1 = int(caps[j]), int(caps1[j])
            if self.track_positions:
                idx_j = idx_slab[int(off_i[j]): int(off_i[j + 1])].view(B, H_kv, c1)
                self.cur_pos[l] = (torch.gather(self.cur_pos[l], 2, idx_j[:, :, :c].long()) if c
                                   else self.cur_pos[l][:, :, :0])
            rows = c + S_w
            self.held[l] = _Held(int(th[7, j]), int(th[8, j]), int(th[9, j]), [H_kv * rows * d, rows * d, d], c,
                                 (k_slab, v_slab, i_slab), None)
            self.held[l].views = (k_slab, v_slab, i_slab, int(off_kv[j]), int(off_i[j]), c1)
            self.cur_len[l] = keep[l]
        return budgets

    def _layer_views(self, l: int):
        B, H_q, H_kv, S_w, d, N, dtype, dev = self._geom
        h = self.held[l]
        if len(h.views) == 3:                         # still the caller's tensors and the full indicator
            return h.views
        k_slab, v_slab, i_slab, o_kv, o_i, c1 = h.views
        rows = h.cap + S_w
        n_kv = B * H_kv * rows * d
        return (k_slab[o_kv: o_kv + n_kv].view(B, H_kv, rows, d), v_slab[o_kv: o_kv + n_kv].view(B, H_kv, rows, d),
                i_slab[o_i: o_i + B * H_kv * c1].view(B, H_kv, c1))

    def result(self) -> PassResult:
        """The caches, indicators and (if tracked) original positions after the stages so far."""
        torch.cuda.synchronize()
        m = self.m
        views = [self._layer_views(l) for l in range(m)]
        idx_final = [p.to(torch.int32) if p is not None else None for p in self.cur_pos]
        return PassResult(self.budgets, self.cur_len[:m].copy(), self.pref[:, :m].copy(), self.hv[:, :m].copy(), [],
                          idx_final, [t[0] for t in views], [t[1] for t in views], [t[2] for t in views],
                          list(self.stage_budgets))


class DeviceCascade:
    """Alg. 1 with nothing read back between the stages: `admit` scores layer m, the budgets
    B^(m) of the layers seen so far are computed on the device (cake_plan_eviction over m + 1
    layers with the previous stage's keep counts as current lengths), and every layer is
    re-evicted from its previous compacted cache into the other of two output pools
    (cake_evict_planned with the earlier layers flagged as compacted).  The output tables and keep
    counts of one stage's plan are handed to the next stage as device data.  Layers admitted while
    everything still fits are copied whole.  Same caches and budgets as CascadeSession (tested);
    original positions are not tracked.  The host waits once, in `result`."""

    def __init__(self, n_layers: int, total_budget: int, params=None):
        self.L, self.total_budget = int(n_layers), int(total_budget)
        self.params = params if params is not None else C.make_params()
        self.m = 0
        self._geom = None

    def _setup(self, q_win, k):
        B, H_q, S_w, d = q_win.shape
        H_kv, N = k.shape[1], k.shape[2]
        dev, dt = k.device, k.dtype
        self._geom = (B, H_q, H_kv, S_w, d, N, dt, dev)
        L = self.L
        self.shape1 = C.make_shape(B, 1, H_q, H_kv, d, N, S_w, dt)
        self.ws1 = torch.empty(C.cake_workspace_bytes(self.shape1), dtype=torch.uint8, device=dev)
        self.pref_all = torch.zeros(B, L, dtype=torch.float64, device=dev)    # every layer's preference, [B, L]
        self.hv_all = torch.zeros(B, L, 2, dtype=torch.float64, device=dev)
        self.pref1 = torch.zeros(B, dtype=torch.float64, device=dev)          # the admitted layer's, [B, 1]
        self.hv1 = torch.zeros(B, 2, dtype=torch.float64, device=dev)
        self.pref_stage = torch.zeros(B * L, dtype=torch.float64, device=dev) # [B, m + 1] contiguous for the plan
        self.cur = torch.full((L, B), N - S_w, dtype=torch.int32, device=dev) # current evictable lengths
        self.status = torch.zeros(B, dtype=torch.int32, device=dev)
        self.shapes = [C.make_shape(B, m + 1, H_q, H_kv, d, N, S_w, dt) for m in range(L)]
        self.layouts = [C.cake_plan_layout(sh) for sh in self.shapes]
        self.plans = [torch.zeros(C.cake_plan_bytes(self.shapes[-1]), dtype=torch.uint8, device=dev) for _ in range(2)]
        # A stage's outputs: layer l holds [B, H_kv, cap_l + S_w, d] with cap_l = max_b keep, and
        # sum_l (keep[l, b] + S_w) <= min(total_budget, (m + 1) N) for every sequence b
        rows = B * min(self.total_budget, L * N)
        bh = B * H_kv
        self.pools = [dict(k=torch.empty(bh * rows * d, dtype=dt, device=dev), v=torch.empty(bh * rows * d, dtype=dt, device=dev),
                           idx=torch.empty(bh * rows, dtype=torch.int32, device=dev),
                           ind=torch.empty(bh * rows, dtype=torch.float32, device=dev)) for _ in range(2)]
        # one pinned row per stage: the host never waits for the device here, so a staging row must
        # not be written again while its upload may still be pending
        self.new_host = torch.zeros(L, 6, dtype=torch.int64).pin_memory()
        self.new_ptrs = torch.zeros(6, dtype=torch.int64, device=dev)         # q, k, indicator tables of the scores; k, v, ind of the layer
        self.inputs = torch.zeros(4, L, dtype=torch.int64, device=dev)        # rows: (unused), K, V, indicator tables of all layers
        self.alive = []

    def _part(self, plan: torch.Tensor, m: int, name: str, dtype, count: int) -> torch.Tensor:
        off = self.layouts[m][name]
        size = torch.empty(0, dtype=dtype).element_size()
        return plan[off: off + count * size].view(dtype)

    def admit(self, q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, indicator_out: Optional[torch.Tensor] = None) -> None:
        assert self.m < self.L, "every layer has been admitted"
        if self._geom is None:
            self._setup(q_win, k)
        B, H_q, H_kv, S_w, d, N, dt, dev = self._geom
        assert tuple(q_win.shape) == (B, H_q, S_w, d) and tuple(k.shape) == (B, H_kv, N, d) and v.shape == k.shape
        assert _strides3(v) == _strides3(k)
        m, n = self.m, self.m + 1
        ind = indicator_out if indicator_out is not None else torch.empty(B, H_kv, N - S_w, dtype=torch.float32, device=dev)
        self.alive = [q_win, k, v, ind] + self.alive[:4]                     # this stage's and the previous stage's inputs
        host = self.new_host[m]
        host.numpy()[:] = (q_win.data_ptr(), k.data_ptr(), ind.data_ptr(), k.data_ptr(), v.data_ptr(), ind.data_ptr())
        self.new_ptrs.copy_(host, non_blocking=True)
        self.inputs[1:4, m].copy_(self.new_ptrs[3:6])
        C.cake_window_scores(self.shape1, self.params, self.new_ptrs[0:1], self.new_ptrs[1:2], _strides3(q_win), _strides3(k),
                             self.new_ptrs[2:3], self.ws1)
        C.cake_layer_preference(self.shape1, self.params, self.ws1, self.pref1, self.hv1)
        self.pref_all[:, m].copy_(self.pref1)
        self.hv_all[:, m].copy_(self.hv1)
        stage_pref = self.pref_stage[: B * n].view(B, n)
        stage_pref.copy_(self.pref_all[:, :n])
        shape, plan, pool = self.shapes[m], self.plans[m & 1], self.pools[m & 1]
        C.cake_plan_eviction(shape, stage_pref, self.total_budget, self.cur, pool["idx"], pool["k"], pool["v"], pool["ind"],
                             plan, self.status)
        C.cake_evict_planned(shape, self.inputs[3], self.inputs[1], self.inputs[2], _strides3(k), plan,
                             compacted=[1] * m + [0])
        # the next stage starts from this stage's outputs: its four tables sit one after the other in the plan
        self.inputs[:, :n].copy_(self._part(plan, m, "idx", torch.int64, 4 * n).view(4, n))
        self.cur[:n].copy_(self._part(plan, m, "keep", torch.int32, n * B).view(n, B))
        self.m = n

    def result(self) -> PassResult:
        """Budgets, keep counts and the final caches (views into the last stage's pool)."""
        torch.cuda.synchronize()
        B, H_q, H_kv, S_w, d, N, dt, dev = self._geom
        m = self.m
        plan, pool = self.plans[(m - 1) & 1], self.pools[(m - 1) & 1]
        if int(self.status.max().item()) != 0:
            raise C.CakeError(-1, "a layer preference is NaN, negative or infinite")
        budgets, keep, _, _ = C.plan_fields(plan.cpu(), m, B)
        caps = keep.max(axis=1).astype(np.int64)
        k_out, v_out, ind_out, idx = [], [], [], []
        o_kv = o_i = 0
        bh = B * H_kv
        for l in range(m):
            c = int(caps[l])
            n_kv, n_i = bh * (c + S_w) * d, bh * c
            k_out.append(pool["k"][o_kv: o_kv + n_kv].view(B, H_kv, c + S_w, d))
            v_out.append(pool["v"][o_kv: o_kv + n_kv].view(B, H_kv, c + S_w, d))
            ind_out.append(pool["ind"][o_i: o_i + n_i].view(B, H_kv, c))
            idx.append(None)
            o_kv += n_kv
            o_i += n_i
        return PassResult(budgets, keep, self.pref_all[:, :m].cpu().numpy(), self.hv_all[:, :m].cpu().numpy(), [], idx, k_out,
                          v_out, ind_out)


@dataclass
class QuantizedCache:
    """Retained prefix rows of every layer in b-bit codes (cake_quantize_kv); per layer tensors."""
    bits: int
    k_codes: List[torch.Tensor]     # [B, H_kv, cap_l, d*bits/8] uint8
    k_scale: List[torch.Tensor]     # [B, H_kv, ceil(cap_l/32), d] f32
    k_zero: List[torch.Tensor]
    v_codes: List[torch.Tensor]     # [B, H_kv, cap_l, d*bits/8] uint8
    v_scale: List[torch.Tensor]     # [B, H_kv, cap_l, d/32] f32
    v_zero: List[torch.Tensor]


class CacheQuantizer:
    """Buffers and the one call that store a pass's retained rows in 2, 4 or 8 bits."""

    def __init__(self, result: PassResult, window: int, bits: int):
        self.bits, self.S_w = int(bits), int(window)
        self.keep = np.asarray(result.keep, dtype=np.int64)
        self.L, self.B = self.keep.shape
        k0 = result.k_out[0]
        self.H_kv, self.d, dev = k0.shape[1], k0.shape[3], k0.device
        self.k_hat, self.v_hat = result.k_out, result.v_out
        self.shape = C.make_shape(self.B, self.L, self.H_kv, self.H_kv, self.d, self.S_w + 1, self.S_w, k0.dtype)
        caps = [int(self.keep[l].max()) for l in range(self.L)]
        mk = lambda shp, dt: [torch.empty(self.B, self.H_kv, *shp(c), dtype=dt, device=dev) for c in caps]
        row_bytes = self.d * self.bits // 8
        self.out = QuantizedCache(
            self.bits,
            mk(lambda c: (max(c, 1), row_bytes), torch.uint8), mk(lambda c: (max(-(-c // 32), 1), self.d), torch.float32),
            mk(lambda c: (max(-(-c // 32), 1), self.d), torch.float32),
            mk(lambda c: (max(c, 1), row_bytes), torch.uint8), mk(lambda c: (max(c, 1), self.d // 32), torch.float32),
            mk(lambda c: (max(c, 1), self.d // 32), torch.float32))
        self.tbl = [C.ptr_table(t) for t in (self.k_hat, self.v_hat, self.out.k_codes, self.out.k_scale, self.out.k_zero,
                                             self.out.v_codes, self.out.v_scale, self.out.v_zero)]
        self.strides = [_strides3(t) for t in self.k_hat]
        self.keep_flat = [int(x) for x in self.keep.reshape(-1)]

    def run(self, stream=None) -> QuantizedCache:
        C.cake_quantize_kv(self.shape, self.bits, self.tbl[0], self.tbl[1], self.strides, self.keep_flat, *self.tbl[2:],
                           stream)
        return self.out


class DecodeCache:
    """The evicted caches of a prompt during generation (implementation appendix, decoding branch):
    every layer stays at the budget the prefill pass gave it.  `step(layer, q_new, k_new, v_new)`
    appends the token's key and value, lets cake_decode_update fold the new query's pooled
    attention into the stored indicator and evicts one scored row per head with the library's
    top-k and compaction (k = cur_len), so the layer returns to its size.  Buffer handling
    (appending a row, the zero for the row that leaves the window) is plain torch."""

    def __init__(self, result: PassResult, n_q_heads: int, window: int, params=None):
        self.params = params if params is not None else C.make_params()
        self.S_w, self.H_q = int(window), int(n_q_heads)
        self.k = [t for t in result.k_out]                 # [B, H_kv, cap_l + S_w, d]
        self.v = [t for t in result.v_out]
        self.cur_len = np.asarray(result.keep, dtype=np.int64).copy()          # [L, B]
        self.L, self.B = self.cur_len.shape
        self.ind = []
        for l in range(self.L):
            cap = int(self.cur_len[l].max())
            self.ind.append(result.ind_out[l][:, :, :cap].contiguous() if cap else
                            result.ind_out[l][:, :, :0].contiguous())
        self._ws = {}
        self._tbl = None
        self._step = 0

    def step(self, layer: int, q_new: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor) -> None:
        """q_new [B, H_q, d]; k_new, v_new [B, H_kv, d]: the generated token's projections at `layer`."""
        l, S_w, B = layer, self.S_w, self.B
        k_old, v_old, i_old = self.k[l], self.v[l], self.ind[l]
        H_kv, d = k_old.shape[1], k_old.shape[3]
        dev = k_old.device
        cur = self.cur_len[l]
        cap = int(cur.max())
        # ---- append: one more row per sequence; the row that leaves the window starts at 0
        k_in = torch.empty(B, H_kv, cap + S_w + 1, d, dtype=k_old.dtype, device=dev)
        v_in = torch.empty_like(k_in)
        i_in = torch.zeros(B, H_kv, cap + 1, dtype=torch.float32, device=dev)
        k_in[:, :, : cap + S_w] = k_old[:, :, : cap + S_w]
        v_in[:, :, : cap + S_w] = v_old[:, :, : cap + S_w]
        i_in[:, :, :cap] = i_old[:, :, :cap]
        if B == 1:
            k_in[:, :, cap + S_w] = k_new
            v_in[:, :, cap + S_w] = v_new
        else:
            for b in range(B):
                n_b = int(cur[b]) + S_w
                k_in[b, :, n_b] = k_new[b]
                v_in[b, :, n_b] = v_new[b]
                i_in[b, :, int(cur[b]):] = 0.0
        cur1 = [int(c) + 1 for c in cur]
        keep = [int(c) for c in cur]
        shape = C.make_shape(B, 1, self.H_q, H_kv, d, cap + S_w + 1, S_w, k_old.dtype)
        key = (B, H_kv, d, cap, str(k_old.dtype))
        if key not in self._ws:
            self._ws = {key: torch.empty(C.cake_workspace_bytes(shape), dtype=torch.uint8, device=dev)}
        ws = self._ws[key]
        q_new = q_new.contiguous()
        idx = torch.zeros(B, H_kv, max(cap, 1), dtype=torch.int32, device=dev)
        k_out = torch.empty(B, H_kv, cap + S_w, d, dtype=k_old.dtype, device=dev)
        v_out = torch.empty_like(k_out)
        i_out = torch.empty(B, H_kv, max(cap, 1), dtype=torch.float32, device=dev)
        # ---- all pointer tables of the step in one upload (two pinned copies used in turn: the
        # step before last has certainly run, each step's kernels are ordered after its upload)
        if self._tbl is None:
            self._tbl = ([torch.zeros(8, dtype=torch.int64).pin_memory() for _ in range(4)],
                         [torch.zeros(8, dtype=torch.int64, device=dev) for _ in range(4)])
        slot = self._step & 3
        if slot == 0 and self._step:
            torch.cuda.current_stream().synchronize()       # the staging copies are about to be reused
        self._step += 1
        host, tbl = self._tbl[0][slot], self._tbl[1][slot]
        th = host.numpy()
        th[:] = [q_new.data_ptr(), k_in.data_ptr(), v_in.data_ptr(), i_in.data_ptr(), idx.data_ptr(), k_out.data_ptr(),
                 v_out.data_ptr(), i_out.data_ptr()]
        tbl.copy_(host, non_blocking=True)
        st = [_strides3(k_in)]
        C.cake_decode_update(shape, self.params, tbl[0:1], [q_new.stride(0), q_new.stride(1)], tbl[1:2], st, cur1,
                             tbl[3:4], ws)
        # ---- evict one scored row per head: back to cur rows
        C.cake_select_topk(shape, tbl[3:4], cur1, keep, tbl[4:5])
        C.cake_compact_kv(shape, tbl[1:2], tbl[2:3], st, cur1, keep, tbl[4:5], tbl[3:4], tbl[5:6], tbl[6:7], tbl[7:8])
        self.k[l], self.v[l], self.ind[l] = k_out, v_out, i_out[:, :, :cap]
        self.last_idx = idx
        self._keep_alive = (q_new, k_in, v_in, i_in)       # until the kernels have run


class DecodeSlots:
    """The evicted caches of a prompt during generation, kept in place (cake_decode_step): every
    layer's K and V sit in fixed slots, a per-head list gives the logical order, and a generated
    token costs one key/value row write per head plus the indicator update.  All buffers, pointer
    tables and the workspace are made once here; `step` allocates nothing."""

    def __init__(self, result: PassResult, n_q_heads: int, window: int, params=None):
        self.params = params if params is not None else C.make_params()
        self.S_w, self.H_q = int(window), int(n_q_heads)
        keep = np.asarray(result.keep, dtype=np.int64)                       # [L, B]
        self.L, self.B = keep.shape
        k0 = result.k_out[0]
        self.H_kv, self.d, self.dtype, dev = k0.shape[1], k0.shape[3], k0.dtype, k0.device
        self.cap = [int(keep[l].max()) for l in range(self.L)]
        self.k, self.v, self.ind, self.order, self.state = [], [], [], [], []
        for l in range(self.L):
            cap, rows = self.cap[l], self.cap[l] + self.S_w + 1
            k = torch.zeros(self.B, self.H_kv, rows, self.d, dtype=self.dtype, device=dev)
            v = torch.zeros_like(k)
            ind = torch.zeros(self.B, self.H_kv, cap + 1, dtype=torch.float32, device=dev)
            order = torch.arange(rows, dtype=torch.int32, device=dev).repeat(self.B, self.H_kv, 1).contiguous()
            state = torch.zeros(self.B, self.H_kv, 4, dtype=torch.int32, device=dev)
            for b in range(self.B):
                n_b = int(keep[l, b])
                k[b, :, : n_b + self.S_w] = result.k_out[l][b, :, : n_b + self.S_w]
                v[b, :, : n_b + self.S_w] = result.v_out[l][b, :, : n_b + self.S_w]
                ind[b, :, :n_b] = result.ind_out[l][b, :, :n_b]
                state[b, :, 0] = n_b
                state[b, :, 1] = n_b + self.S_w                               # first unused slot
            self.k.append(k); self.v.append(v); self.ind.append(ind); self.order.append(order); self.state.append(state)
        self.tbl = {name: C.ptr_table(getattr(self, name)) for name in ("k", "v", "ind", "order", "state")}
        rows_max = max(self.cap) + self.S_w + 1
        self.shape1 = C.make_shape(self.B, 1, self.H_q, self.H_kv, self.d, rows_max, self.S_w, self.dtype)
        self.ws = torch.empty(C.cake_decode_step_workspace_bytes(self.shape1), dtype=torch.uint8, device=dev)
        self.slot_strides = [_strides3(t) for t in self.k]
        self._ws_all = None

    def step(self, layer: int, q_new: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor) -> None:
        """q_new [B, H_q, d]; k_new, v_new [B, H_kv, d]: the generated token's projections at `layer`."""
        l = layer
        assert q_new.stride(2) == 1 and k_new.stride(2) == 1 and v_new.stride() == k_new.stride()
        C.cake_decode_step(self.shape1, self.params, q_new, [0, q_new.stride(0), q_new.stride(1)], k_new, v_new,
                           [0, k_new.stride(0), k_new.stride(1)], self.tbl["k"][l:l + 1], self.tbl["v"][l:l + 1],
                           [self.slot_strides[l]], self.tbl["ind"][l:l + 1], self.tbl["order"][l:l + 1],
                           self.tbl["state"][l:l + 1], [self.cap[l]], self.ws)

    def step_all(self, q_new: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor) -> None:
        """The maintenance of one generated token for every layer in one call per 32 layers, for a
        caller that keeps the token's projections of all layers until its forward pass is over.
        q_new [L, B, H_q, d]; k_new, v_new [L, B, H_kv, d].  Same result as `step` layer by layer."""
        assert q_new.stride(3) == 1 and k_new.stride(3) == 1 and v_new.stride() == k_new.stride()
        per_call = 32
        if self._ws_all is None:
            n = min(per_call, self.L)
            self._shape_all = C.make_shape(self.B, n, self.H_q, self.H_kv, self.d, max(self.cap) + self.S_w + 1, self.S_w,
                                           self.dtype)
            self._ws_all = torch.empty(C.cake_decode_step_workspace_bytes(self._shape_all), dtype=torch.uint8,
                                       device=self.ws.device)
        for l0 in range(0, self.L, per_call):
            l1 = min(l0 + per_call, self.L)
            shape = self._shape_all if l1 - l0 == self._shape_all.n_layers else C.make_shape(
                self.B, l1 - l0, self.H_q, self.H_kv, self.d, max(self.cap) + self.S_w + 1, self.S_w, self.dtype)
            C.cake_decode_step(shape, self.params, q_new[l0:l1], list(q_new.stride()[:3]), k_new[l0:l1], v_new[l0:l1],
                               list(k_new.stride()[:3]), self.tbl["k"][l0:l1], self.tbl["v"][l0:l1],
                               self.slot_strides[l0:l1], self.tbl["ind"][l0:l1], self.tbl["order"][l0:l1],
                               self.tbl["state"][l0:l1], self.cap[l0:l1], self._ws_all)

    def logical(self, layer: int, b: int):
        """(K, V [H_kv, cur + S_w, d], indicator [H_kv, cur], evicted logical index [H_kv]) of one
        sequence in logical order: the view the method describes.  Inspection only."""
        st = self.state[layer][b].cpu().numpy()
        cur = int(st[0, 0])
        order = self.order[layer][b, :, : cur + self.S_w].long()
        gather = order[:, :, None].expand(-1, -1, self.d)
        return (torch.gather(self.k[layer][b], 1, gather), torch.gather(self.v[layer][b], 1, gather),
                self.ind[layer][b, :, :cur], st[:, 2].copy())
