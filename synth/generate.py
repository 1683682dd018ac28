"""Seeded synthetic Q/K/V for the prefill eviction pass.

The paper evaluates on long-context benchmark prompts run through trained models;
neither is available here, so these tensors stand in for them.  They have the
shapes of the paper's GQA models (32 layers, 32 query / 8 KV heads, head_dim 128)
and imitate the attention structures the paper describes: layers whose attention
is broad and layers whose attention is peaked (a per-layer logit temperature),
attention sinks at the first positions, a recency band, heavy-hitter keys, and
heavy hitters whose weight drifts across the observation window.

Structure is planted through reserved orthonormal directions e_1..e_4 per
(layer, KV head).  The random parts of Q and K are projected off their span, so a
key row that carries `beta * e_i` gains exactly `beta * c_r` logits for a window
query that carries `sqrt(d) * c_r * e_i` (after the 1/sqrt(d) softmax scale).

Everything is drawn from `torch.Generator`s seeded `1000*config + 10*layer + b`.
The caller generates once and hands identical bits to the GPU path and to the
CPU oracle.  This module holds no arithmetic of the eviction method itself.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Dict, List, Optional

import torch


@dataclass(frozen=True)
class CakeConfig:
    cid: int
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int          # N: rows of K/V per head, window included
    window: int           # S_w
    total_budget: int     # B_total per KV head, summed over layers, windows included
    dtype: str            # "bf16" | "f32"
    batch: int
    temperature: str      # "tiny" | "uniform" | "geometric"
    sink: bool
    band: bool
    heavy: str            # "none" | "static8" | "drift32"

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def prefix_len(self) -> int:
        return self.seq_len - self.window

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    def scaled(self, **kw) -> "CakeConfig":
        """A reduced or altered copy (tests use smaller N / fewer layers)."""
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[int, CakeConfig] = {
    1: CakeConfig(1, "tiny", 2, 4, 2, 64, 1024, 32, 256, "f32", 1, "tiny", False, False, "static8"),
    2: CakeConfig(2, "llama8b-8k", 32, 32, 8, 128, 8192, 32, 32 * 1024, "bf16", 1, "uniform", True, True, "none"),
    3: CakeConfig(3, "llama8b-32k", 32, 32, 8, 128, 32768, 32, int(0.032 * 32768 * 32), "bf16", 1,
                  "uniform", True, True, "drift32"),
    4: CakeConfig(4, "llama8b-128k", 32, 32, 8, 128, 131072, 64, 32 * 2048, "bf16", 1, "uniform", True, True, "none"),
    5: CakeConfig(5, "gqa5-64L-b4", 64, 40, 8, 128, 32768, 32, 64 * 1024, "bf16", 4, "geometric", True, True, "none"),
}

SINK_LEN = 4
SINK_BETA = 4.0
BAND_WIDTH = 64
BAND_BETA = 2.0
HEAVY_STATIC_BETA = 3.0
HEAVY_DRIFT_BETA = 4.0


def _seed(cfg: CakeConfig, layer: int, b: int) -> int:
    return 1000 * cfg.cid + 10 * layer + b


def layer_temperature(cfg: CakeConfig, layer: int, b: int) -> float:
    """Multiplier on the random part of the window queries of (layer, sequence b)."""
    if cfg.temperature == "tiny":
        return 4.0 if layer == 1 else 1.0
    if cfg.temperature == "uniform":
        g = torch.Generator().manual_seed(1000 * cfg.cid + 7)
        t = 0.5 + 3.5 * torch.rand(max(cfg.n_layers, 64), generator=g, dtype=torch.float64)
        return float(t[layer])
    if cfg.temperature == "geometric":
        g = torch.Generator().manual_seed(1000 * cfg.cid + 7 + b)
        u = 0.8 + 0.45 * torch.rand(max(cfg.n_layers, 64), generator=g, dtype=torch.float64)
        frac = layer / max(cfg.n_layers - 1, 1)
        return float(0.25 * (16.0 ** frac) * u[layer])
    raise ValueError(cfg.temperature)


def _orthonormal_directions(h_kv: int, d: int, gen: torch.Generator, device) -> torch.Tensor:
    raw = torch.randn(h_kv, d, 4, generator=gen, device=device, dtype=torch.float32)
    q, _ = torch.linalg.qr(raw.double().cpu())          # [h_kv, d, 4], orthonormal columns
    return q.transpose(1, 2).contiguous().float().to(device)  # [h_kv, 4, d]


def _project_off(x: torch.Tensor, e: torch.Tensor) -> torch.Tensor:
    """Remove from the rows of x [h, n, d] their components along e [h, 4, d]."""
    coeff = torch.bmm(x, e.transpose(1, 2))             # [h, n, 4]
    return x - torch.bmm(coeff, e)


def make_layer(cfg: CakeConfig, layer: int, b: int = 0, device="cpu") -> dict:
    """Q_w [H_q,S_w,d], K [H_kv,N,d], V [H_kv,N,d] in cfg's dtype, plus metadata."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev).manual_seed(_seed(cfg, layer, b))
    cgen = torch.Generator().manual_seed(_seed(cfg, layer, b) + 500_000)   # positions: host draws
    hq, hkv, d, n, sw, g = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.seq_len, cfg.window, cfg.group
    n_p = n - sw
    rootd = math.sqrt(d)

    e = _orthonormal_directions(hkv, d, gen, dev)                          # [hkv,4,d]
    q0 = torch.randn(hq, sw, d, generator=gen, device=dev, dtype=torch.float32)
    k = torch.randn(hkv, n, d, generator=gen, device=dev, dtype=torch.float32)
    v = torch.randn(hkv, n, d, generator=gen, device=dev, dtype=torch.float32)

    k = _project_off(k, e)
    e_q = e.repeat_interleave(g, dim=0)                                    # [hq,4,d]
    q = _project_off(q0, e_q) * layer_temperature(cfg, layer, b)

    # per-row coefficient of each reserved direction in the window queries
    coeff = torch.zeros(sw, 4, device=dev, dtype=torch.float32)
    ramp = torch.arange(sw, device=dev, dtype=torch.float32) / max(sw - 1, 1)
    meta = {"temperature": layer_temperature(cfg, layer, b), "heavy": None}

    if cfg.heavy == "static8":
        pos = torch.randperm(n_p, generator=cgen)[:8].sort().values
        coeff[:, 0] = 1.0
        k[:, pos.to(dev), :] += HEAVY_STATIC_BETA * e[:, 0:1, :]
        meta["heavy"] = pos.unsqueeze(0).expand(hkv, -1).clone()
    elif cfg.heavy == "drift32":
        coeff[:, 0] = ramp            # boost rises 0 -> beta across the window
        coeff[:, 3] = 1.0 - ramp      # boost falls beta -> 0
        allpos = []
        for h in range(hkv):
            pos = torch.randperm(n_p - SINK_LEN - BAND_WIDTH, generator=cgen)[:32] + SINK_LEN
            k[h, pos[:16].to(dev), :] += HEAVY_DRIFT_BETA * e[h, 0, :]
            k[h, pos[16:].to(dev), :] += HEAVY_DRIFT_BETA * e[h, 3, :]
            allpos.append(pos.sort().values)
        meta["heavy"] = torch.stack(allpos)
    if cfg.sink:
        coeff[:, 1] = 1.0
        k[:, :SINK_LEN, :] += SINK_BETA * e[:, 1:2, :]
    if cfg.band:
        coeff[:, 2] = 1.0
        lo = max(n_p - BAND_WIDTH, 0)
        k[:, lo:n_p, :] += BAND_BETA * e[:, 2:3, :]

    q = q + rootd * torch.einsum("ri,hid->hrd", coeff, e_q)
    dt = cfg.torch_dtype
    return {"q_win": q.to(dt).contiguous(), "k": k.to(dt).contiguous(), "v": v.to(dt).contiguous(), "meta": meta}


def make_config_inputs(cfg: CakeConfig, device="cpu", layers: Optional[List[int]] = None) -> dict:
    """All (or the listed) layers of a config as stacked tensors.

    Returns q_win [L,B,H_q,S_w,d], k and v [L,B,H_kv,N,d]; `meta[l][b]` per layer/sequence.
    """
    layers = list(range(cfg.n_layers)) if layers is None else list(layers)
    dt, dev = cfg.torch_dtype, torch.device(device)
    nl, bsz = len(layers), cfg.batch
    q = torch.empty(nl, bsz, cfg.n_q_heads, cfg.window, cfg.head_dim, dtype=dt, device=dev)
    k = torch.empty(nl, bsz, cfg.n_kv_heads, cfg.seq_len, cfg.head_dim, dtype=dt, device=dev)
    v = torch.empty_like(k)
    meta = []
    for i, layer in enumerate(layers):
        row = []
        for b in range(bsz):
            one = make_layer(cfg, layer, b, device=dev)
            q[i, b], k[i, b], v[i, b] = one["q_win"], one["k"], one["v"]
            row.append(one["meta"])
            del one
        meta.append(row)
    return {"q_win": q, "k": k, "v": v, "meta": meta, "layers": layers}
