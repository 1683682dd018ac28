#!/usr/bin/env python3
"""Benchmark of the CAKE prefill eviction pass on one MI355X.

One "step" is the whole hot path over one prompt's resident K/V: window scores for all
layers, layer preferences, Eq. 7 allocation and output placement on the device, per-head
top-k and K/V compaction for all layers; nothing inside a step waits for the GPU.  Inputs are synthetic
(synth/generate.py) and already resident in HBM when the timed region starts.

Prints ONE JSON line.  `value` = B*N*L / seconds per step (prefix tokens x layers per second).
`roofline` describes the dominant kernel, timed live with HIP events inside the timed region.
`cpu_baseline` times the fp64 NumPy oracle on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
MFMA_F32_PEAK_TFLOPS = 157.3


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="synthetic config id (4 = 128K context, the headline)")
    ap.add_argument("--layers", type=int, default=0, help="override layer count (0 = the config's)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--row-lse", action="store_true",
                    help="variant: hand the window rows' log-sum-exp to the library (cake_window_scores_lse), "
                         "as a prefill attention kernel would; the scores then read K once")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy and a sparse 256-byte-row gather four times each "
                         "(references for the HBM byte counters)")
    ap.add_argument("--flush-cache", action="store_true",
                    help="overwrite a 1 GiB buffer before every step (outside the per-step event bracket), so that small "
                         "configs start every pass with cold L2 and last-level cache; adds ms_per_step_flushed")
    ap.add_argument("--decode", action="store_true",
                    help="instead of the prefill pass: time the decode-phase cache maintenance of one generated token "
                         "over all layers (in-place step, and the append + compaction form beside it)")
    ap.add_argument("--quantize", type=int, default=0, metavar="BITS",
                    help="instead of the pass: after one pass, time the 2/4/8-bit storage of the retained rows "
                         "(cake_quantize_kv)")
    ap.add_argument("--cascade", action="store_true",
                    help="instead of the one-shot pass: Alg. 1 stage by stage (every admitted layer scored alone, all "
                         "earlier layers re-evicted to their new budgets), same final caches by Thm. 2")
    ap.add_argument("--host-allocation", action="store_true",
                    help="variant: budgets on the host (cake_cascade_allocate) between the scores and EVICT")
    return ap.parse_args()


def cpu_baseline(cfg, layer_inputs, params):
    """Time the oracle on KV heads of layer 0, one after the other for about 12 s (scores, indicator,
    top-k, compaction), plus one allocation; scale to tokens*layers/s by the fraction of a layer done."""
    import numpy as np
    from oracle import cake_oracle as co
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        threads = os.cpu_count() or 1
    p = co.OracleParams(scale=None, gamma=params.gamma, tau1=params.tau1, tau2=params.tau2,
                        var_correction=params.var_correction, pool_kernel=params.pool_kernel,
                        indicator_mode=params.indicator_mode)
    group = cfg.n_q_heads // cfg.n_kv_heads
    q = layer_inputs["q_win"].double().cpu().numpy()
    heads_done, t_total = 0, 0.0
    keep = max(cfg.total_budget // cfg.n_layers - cfg.window, 1)
    budget_s = 12.0          # keep going, head after head (layer 0 again when its heads are used up), for this long
    while t_total <= budget_s:
        g = heads_done % cfg.n_kv_heads
        k_g = layer_inputs["k"][g:g + 1].double().cpu().numpy()
        v_g = layer_inputs["v"][g].double().cpu().numpy()
        t0 = time.perf_counter()
        a_obs = co.observed(co.window_attention(q[g * group:(g + 1) * group], k_g, p.scale), cfg.window)
        ind = co.eviction_indicator(a_obs, group, p)[0]
        co.dispersion(a_obs); co.shift(a_obs, p.var_correction)
        co.evict(k_g[0], v_g, ind, keep + cfg.window, cfg.window)
        t_total += time.perf_counter() - t0
        heads_done += 1
    t0 = time.perf_counter()
    co.cascade_allocate(np.linspace(0.5, 2.0, cfg.n_layers), cfg.total_budget, cfg.window, cfg.seq_len)
    t_alloc = time.perf_counter() - t0
    layer_frac = heads_done / cfg.n_kv_heads
    tokens_layers = cfg.seq_len * layer_frac
    value = tokens_layers / (t_total + t_alloc * layer_frac / cfg.n_layers)
    return {"value": value, "unit": "tokens*layers/s", "cores": int(threads), "kind": "oracle",
            "sample": f"config {cfg.cid} layer 0's inputs, {heads_done} KV-head passes of {cfg.n_kv_heads} per layer (window "
                      f"attention, indicator, H, V, top-k, compaction) in {t_total:.1f} s, plus one {cfg.n_layers}-layer "
                      f"allocation; scaled by the fraction of a layer done"}


def measured_traffic(cfg, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter runs (FETCH_SIZE +
    WRITE_SIZE, scaled by what the same counters read for a plain copy), or None if not measured
    for this workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(path))
        return table[f"config{cfg.cid}"]["kernels"][kernel]["hbm_bytes"]
    except Exception:
        return None


def decode_bench(cake, cfg, ev, steps, warmup):
    """One generated token's cache maintenance in every layer (new query/key/value rows of synthetic
    values), after one prefill pass of the config: microseconds per layer per token on the stream."""
    import torch
    res = ev.run()
    torch.cuda.synchronize()
    dev = ev.dev
    g = torch.Generator().manual_seed(0)
    qn = torch.randn(cfg.batch, cfg.n_q_heads, cfg.head_dim, generator=g).to(cfg.torch_dtype).to(dev)
    kn = torch.randn(cfg.batch, cfg.n_kv_heads, cfg.head_dim, generator=g).to(cfg.torch_dtype).to(dev)
    L = cfg.n_layers
    out = {}
    for name, cache in (("in_place_step", cake.DecodeSlots(res, cfg.n_q_heads, cfg.window)),
                        ("append_and_compact", cake.DecodeCache(res, cfg.n_q_heads, cfg.window))):
        for _ in range(warmup):
            for l in range(L):
                cache.step(l, qn, kn, kn)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            for l in range(L):
                cache.step(l, qn, kn, kn)
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        out[name] = {"us_per_layer_stream": e0.elapsed_time(e1) / steps / L * 1e3, "us_per_layer_wall": wall / L * 1e6,
                     "ms_per_token_wall": wall * 1e3}
    # all layers in one call, for a caller that keeps the token's projections until its forward pass is over
    cache = cake.DecodeSlots(res, cfg.n_q_heads, cfg.window)
    q_all = qn[None].expand(L, -1, -1, -1).contiguous()
    k_all = kn[None].expand(L, -1, -1, -1).contiguous()
    for _ in range(warmup):
        cache.step_all(q_all, k_all, k_all)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        cache.step_all(q_all, k_all, k_all)
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    out["in_place_all_layers_one_call"] = {"us_per_layer_stream": e0.elapsed_time(e1) / steps / L * 1e3,
                                           "us_per_layer_wall": wall / L * 1e6, "ms_per_token_wall": wall * 1e3}
    print(json.dumps({"metric": "decode cache maintenance per generated token", "unit": "us per layer", "n_gpus": 1,
                      "value": out["in_place_step"]["us_per_layer_stream"], "higher_is_better": False, "steps": steps,
                      "warmup": warmup, "dtype": cfg.dtype, "data": "synthetic",
                      "config": {"workload": f"config {cfg.cid} ({cfg.name}) after one prefill pass: {L} layers, rows per head "
                                             f"{int(res.keep.min())}..{int(res.keep.max())} + window {cfg.window}"},
                      "variants": out}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py measures one GPU only: this build has no multi-GPU path (asked for --gpus {args.gpus}).",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (torch.cuda.is_available() is False).", file=sys.stderr)
        sys.exit(2)
    from synth import CONFIGS, make_layer
    import paper_2503_12491_amd as cake
    from paper_2503_12491_amd import _ffi
    if not os.path.exists(_ffi.LIB_PATH):
        from paper_2503_12491_amd.build import build
        build()

    cfg = CONFIGS[args.config]
    if args.layers:
        cfg = cfg.scaled(n_layers=args.layers, total_budget=cfg.total_budget // cfg.n_layers * args.layers)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L, B = cfg.n_layers, cfg.batch
    dt = cfg.torch_dtype
    q_all = torch.empty(L, B, cfg.n_q_heads, cfg.window, cfg.head_dim, dtype=dt, device=dev)
    k_all = torch.empty(L, B, cfg.n_kv_heads, cfg.seq_len, cfg.head_dim, dtype=dt, device=dev)
    v_all = torch.empty_like(k_all)
    for l in range(L):
        for b in range(B):
            one = make_layer(cfg, l, b, device=dev)
            q_all[l, b], k_all[l, b], v_all[l, b] = one["q_win"], one["k"], one["v"]
            del one
    torch.cuda.synchronize()
    params = cake.make_params()
    row_lse = None
    if args.row_lse:
        # stand-in for the normalisers a prefill attention kernel returns: torch, one layer at a time
        row_lse = []
        G = cfg.n_q_heads // cfg.n_kv_heads
        pos_q = cfg.prefix_len + torch.arange(cfg.window, device=dev)
        for l in range(L):
            qf = q_all[l].float().view(B, cfg.n_kv_heads, G * cfg.window, cfg.head_dim) * cfg.head_dim ** -0.5
            s_ = torch.matmul(qf, k_all[l].float().transpose(-1, -2)).view(B, cfg.n_q_heads, cfg.window, cfg.seq_len)
            tail = s_[..., cfg.prefix_len:]
            tail.masked_fill_(torch.arange(cfg.prefix_len, cfg.seq_len, device=dev)[None, :] > pos_q[:, None], float("-inf"))
            row_lse.append(torch.logsumexp(s_, dim=-1).contiguous())
            del qf, s_, tail
    ev = cake.EvictionPass([q_all[l] for l in range(L)], [k_all[l] for l in range(L)], [v_all[l] for l in range(L)],
                           cfg.total_budget, params, row_lse=row_lse)

    if args.decode:
        decode_bench(cake, cfg, ev, args.steps, args.warmup)
        return
    if args.quantize:
        res = ev.run()
        torch.cuda.synchronize()
        quant = cake.CacheQuantizer(res, cfg.window, args.quantize)
        for _ in range(args.warmup):
            quant.run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            quant.run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        rows = int(res.keep.sum()) * cfg.n_kv_heads
        eb = 2 if cfg.dtype == "bf16" else 4
        read_b = rows * cfg.head_dim * eb * 2
        write_b = rows * (cfg.head_dim * args.quantize // 8) * 2 + rows * (cfg.head_dim // 32) * 8 + \
            sum(-(-int(k) // 32) for k in res.keep.reshape(-1)) * cfg.n_kv_heads * cfg.head_dim * 8
        print(json.dumps({"metric": f"retained rows quantised to {args.quantize} bits", "value": rows / (ms * 1e-3),
                          "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
                          "higher_is_better": True, "dtype": cfg.dtype, "data": "synthetic",
                          "config": {"workload": f"config {cfg.cid} ({cfg.name}): {rows} retained (head, row) pairs after one pass"},
                          "roofline": {"kernel": "quantize_kv", "bound": "hbm", "achieved": (read_b + write_b) / (ms * 1e-3) / 1e9,
                                       "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                       "frac": (read_b + write_b) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": None}}))
        return
    if args.cascade:
        on_device = not args.host_allocation                 # stages chained on the device

        def one_cascade():
            if not on_device:
                return ev.run_cascade(track_positions=False)
            session = cake.DeviceCascade(L, cfg.total_budget, params)
            for l in range(L):
                session.admit(q_all[l], k_all[l], v_all[l], indicator_out=ev.indicator[l])
            return session
        for _ in range(args.warmup):
            one_cascade()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_cascade()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        how = "stages chained on the device" if on_device else "one host read-back per stage"
        print(json.dumps({"metric": f"prefix tokens*layers/s evicted (config {cfg.cid}, cascade mode)",
                          "value": B * cfg.seq_len * L / (ms * 1e-3), "unit": "tokens*layers/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
                          "dtype": cfg.dtype, "data": "synthetic",
                          "config": {"workload": f"config {cfg.cid} ({cfg.name}): Alg. 1 in {L} stages, {how}"}}))
        return

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        # and a sparse gather of 256-byte rows (every 16th row on average, ascending), the access
        # pattern of the compaction: 2^18 rows of a 1 GiB table -> 64 MiB read, 64 MiB written
        table = src.view(torch.bfloat16).view(-1, 128)
        g = torch.Generator(device="cpu").manual_seed(1)
        rows = torch.sort(torch.randperm(table.shape[0], generator=g)[: 1 << 18]).values.to(dev)
        for _ in range(4):
            picked = table.index_select(0, rows)
        torch.cuda.synchronize()
        del src, dst, table, rows, picked

    for _ in range(args.warmup):
        ev.run()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` passes, per-kernel HIP events on the launch stream ----
    # (libcake is handed torch's current stream, so torch events and the library's own profiling
    # events all sit on the stream the kernels run on)
    cake.cake_profile_enable(True)
    first = "scores_pass1" if not args.row_lse else "scores_import_lse"
    score_names = [first, "scores_combine", "scores_pass2", "pool_indicator"]
    names = score_names + ["layer_preference", "plan_eviction", "select_topk+compact_kv"]
    if args.host_allocation:
        names = score_names + ["layer_preference", "select_topk", "compact_kv"]
    kernel_ms = {n: 0.0 for n in names}
    ne = 6
    e = [[torch.cuda.Event(enable_timing=True) for _ in range(ne)] for _ in range(args.steps)]
    flush_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev) if args.flush_cache else None
    q_str = [q_all[0].stride(i) for i in range(3)]
    k_str = [k_all[0].stride(i) for i in range(3)]
    keep = None
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(args.steps):
        if flush_buf is not None:
            flush_buf.fill_(s & 0xFF)
        e[s][0].record()
        if row_lse is None:
            cake.cake_window_scores(ev.shape, ev.params, ev.tbl_q, ev.tbl_k, q_str, k_str, ev.tbl_ind, ev.workspace)
        else:
            cake.cake_window_scores_lse(ev.shape, ev.params, ev.tbl_q, ev.tbl_k, q_str, k_str, ev.tbl_lse, ev.tbl_ind,
                                        ev.workspace)
        e[s][1].record()
        cake.cake_layer_preference(ev.shape, ev.params, ev.workspace, ev.pref, ev.hv)
        e[s][2].record()
        if args.host_allocation:
            pref, hv = ev.preferences_to_host()
            budgets = ev.allocate(pref)
            keep = cake.cake_keep_counts(budgets, ev.N_p, ev.S_w)
            ev._carve_outputs(keep)
            kk = keep.reshape(-1).tolist()
            e[s][3].record()
            cake.cake_select_topk(ev.shape, ev.tbl_ind, ev._cur_full, kk, ev.tbl_out[0])
            e[s][4].record()
            cake.cake_compact_kv(ev.shape, ev.tbl_k, ev.tbl_v, ev._strides_full, ev._cur_full, kk, ev.tbl_out[0],
                                 ev.tbl_ind, ev.tbl_out[1], ev.tbl_out[2], ev.tbl_out[3])
        else:
            cake.cake_plan_eviction(ev.shape, ev.pref, ev.total_budget, None, ev.pool_idx, ev.pool_k, ev.pool_v,
                                    ev.pool_ind, ev.plan, ev.status)
            e[s][3].record()
            cake.cake_evict_planned(ev.shape, ev.tbl_ind, ev.tbl_k, ev.tbl_v, k_str, ev.plan)
            e[s][4].record()
        e[s][5].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    step_ms = np.array([e[s][0].elapsed_time(e[s][5]) for s in range(args.steps)])
    score_ms = np.array(cake.cake_profile_read())      # averaged by the library over the profiled calls
    for n, ms in zip(score_names, score_ms):
        kernel_ms[n] = float(ms)
    kernel_ms["layer_preference"] = float(np.mean([e[s][1].elapsed_time(e[s][2]) for s in range(args.steps)]))
    if args.host_allocation:
        kernel_ms["select_topk"] = float(np.mean([e[s][3].elapsed_time(e[s][4]) for s in range(args.steps)]))
        kernel_ms["compact_kv"] = float(np.mean([e[s][4].elapsed_time(e[s][5]) for s in range(args.steps)]))
    else:
        kernel_ms["plan_eviction"] = float(np.mean([e[s][2].elapsed_time(e[s][3]) for s in range(args.steps)]))
        kernel_ms["select_topk+compact_kv"] = float(np.mean([e[s][3].elapsed_time(e[s][4]) for s in range(args.steps)]))
        budgets, keep, _, _ = ev.read_plan()
    cake.cake_profile_enable(False)
    if flush_buf is not None:
        # the wall clock contains the flushes: the per-step figure is the mean of the event brackets
        ms_per_step = float(step_ms.mean())
    else:
        ms_per_step = elapsed / args.steps * 1e3
    step_s = ms_per_step * 1e-3
    tokens_layers = B * cfg.seq_len * L
    value = tokens_layers / step_s

    # ---- algorithmic bytes (one read of K, indicator traffic, gathered rows) --------------------
    eb = 2 if cfg.dtype == "bf16" else 4
    k_bytes = tokens_layers * cfg.n_kv_heads * cfg.head_dim * eb                     # one read of K
    n_rows = B * L * cfg.n_kv_heads
    ind_bytes = n_rows * cfg.prefix_len * 4
    kept_rows = int((keep.sum() + L * B * cfg.window) * cfg.n_kv_heads)
    compact_bytes = kept_rows * cfg.head_dim * eb * 2 * 2                            # K and V, read + write
    alg = {"scores_pass1": k_bytes, "scores_import_lse": 0, "scores_pass2": k_bytes + ind_bytes, "pool_indicator": 2 * ind_bytes,
           "select_topk": 4 * ind_bytes, "compact_kv": compact_bytes, "select_topk+compact_kv": 4 * ind_bytes + compact_bytes,
           "scores_combine": 0, "layer_preference": 0, "plan_eviction": 0}
    pass_alg_bytes = k_bytes + ind_bytes * 7 + compact_bytes        # K counted once: the second read is the method's choice
    dominant = max(kernel_ms, key=kernel_ms.get)
    dom_s = kernel_ms[dominant] * 1e-3
    flops_pass = 2.0 * tokens_layers * cfg.n_q_heads * cfg.window * cfg.head_dim   # one logits pass
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS
    achieved = alg[dominant] / dom_s / 1e9
    # The dominant kernel streams K once: its algorithmic bytes over its live duration against the
    # HBM peak.  Its contraction is quoted beside it against the dense MFMA peak of its dtype.
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(cfg, dominant),
                "duration_ms": kernel_ms[dominant]}
    if dominant in ("scores_pass1", "scores_pass2"):
        tf = flops_pass / dom_s / 1e12
        roofline["mfma"] = {"achieved": tf, "peak": mfma_peak, "unit": "TFLOP/s", "frac": tf / mfma_peak}
    score_passes = [n for n in ("scores_pass1", "scores_pass2") if n in kernel_ms]
    extra = {
        "kernel_ms": {n: round(v, 4) for n, v in kernel_ms.items()},
        "ms_per_step_median": float(np.median(step_ms)), "ms_per_step_min": float(step_ms.min()),
        "ms_per_step_event_mean": float(step_ms.mean()),
        "pass_algorithmic_GBps": pass_alg_bytes / step_s / 1e9,
        "pass_hbm_frac": pass_alg_bytes / step_s / 1e9 / HBM_PEAK_GBPS,
        "score_mfma_TFLOPs": {n: flops_pass / (kernel_ms[n] * 1e-3) / 1e12 for n in score_passes},
        "score_mfma_frac": {n: flops_pass / (kernel_ms[n] * 1e-3) / 1e12 / mfma_peak for n in score_passes},
        "host_and_gaps_ms": float(step_ms.mean()) - sum(kernel_ms.values()),
    }
    if flush_buf is not None:
        extra["ms_per_step_flushed"] = float(step_ms.mean())

    out = {
        "metric": "prefix tokens*layers/s evicted at 128K ctx" if cfg.cid == 4 else f"prefix tokens*layers/s evicted (config {cfg.cid})",
        "value": value, "unit": "tokens*layers/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"config {cfg.cid} ({cfg.name}): L={L} H_q={cfg.n_q_heads} H_kv={cfg.n_kv_heads} "
                               f"d={cfg.head_dim} N={cfg.seq_len} S_w={cfg.window} B={B} B_total={cfg.total_budget} "
                               f"one-shot pass" + (", row LSE handed over (K read once)" if args.row_lse else "")
                               + (", budgets on the host" if args.host_allocation else "")
                               + (", caches flushed before every step" if args.flush_cache else ""), "gamma": params.gamma, "tau1": params.tau1, "tau2": params.tau2,
                   "pool_kernel": params.pool_kernel},
        "roofline": roofline, "stages": extra,
    }
    if not args.no_cpu_baseline:
        layer0 = {"q_win": q_all[0, 0], "k": k_all[0, 0], "v": v_all[0, 0]}
        out["cpu_baseline"] = cpu_baseline(cfg, layer0, params)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
