"""Seeded synthetic workloads for the prefill-end retention step.

This module only draws random tensors and tables; it holds none of the method's arithmetic and is
the one piece shared by the HIP path's drivers and the CPU oracle's tests. The paper evaluates on
real 7B-8B backbones and public long-context suites; those models, prompts and compiled tables are
not available here, so every workload is a synthetic stand-in with the backbones' attention shapes
(32 layers, 32 query / 8 KV heads, head_dim 128; 28 layers, 28 / 4 heads), the paper's budgets
(128 / 512 / 1024) and windows (32, 64), and the attention phenomena it names: heavy-tailed and
scale-biased heads (its diagnosis E1), attention sinks and needles (its needle-in-a-haystack test).

Tensors are drawn with ``torch.Generator`` on the device that is asked for; a CPU draw and a GPU draw
of the same workload follow the same recipe but are different samples, so a comparison always copies
one side's tensors to the other.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch

POOL_NONE, POOL_AVG, POOL_MAX = 0, 1, 2


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int          # T, window included
    window: int           # W
    pool: int
    pool_kernel: int
    budget: int           # B per KV head, window included
    n_layers: int
    seed: int
    needles: int = 0          # planted keys per KV head, each 4x a window query row of its group
    sink_scale: float = 0.0   # key 0 multiplied by this (0 = no sink)
    pareto_frac: float = 0.0  # fraction of key rows whose norm is scaled by a Pareto(alpha=2) draw
    head_key_scale: bool = False  # one log-uniform [0.5,4] scale per KV head (scale-biased heads)
    shares: bool = False      # non-uniform per-head budget shares (sum to one per layer)
    gate: bool = False        # 20 x 4 risk-gate table + per-prompt risk bins

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def prefix(self) -> int:
        return self.seq_len - self.window

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def cap(self) -> int:
        """Largest budget one KV head can be handed: the layer total minus every other head's floor W."""
        b_tot = self.budget * self.n_kv_heads
        return min(self.seq_len, b_tot - (self.n_kv_heads - 1) * self.window)

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five configurations the metric is defined on (index = position in the baseline's list).
C1 = Workload("c1_f32_mha4_d64_T1k", "f32", 1, 4, 4, 64, 1024, 32, POOL_AVG, 7, 128, 1, seed=1,
              needles=3, shares=True)
C2 = Workload("c2_bf16_mha32_T4k", "bf16", 1, 32, 32, 128, 4096, 32, POOL_MAX, 7, 512, 1, seed=2,
              sink_scale=8.0)
C3 = Workload("c3_bf16_gqa32x8_T32k_bz16", "bf16", 16, 32, 8, 128, 32768, 32, POOL_AVG, 7, 512, 32,
              seed=3, pareto_frac=0.05, shares=True)
C4 = Workload("c4_bf16_gqa32x8_T128k", "bf16", 1, 32, 8, 128, 131072, 64, POOL_MAX, 7, 512, 32,
              seed=4, needles=16, sink_scale=8.0, shares=True)
C5 = Workload("c5_bf16_gqa28x4_T64k_bz4", "bf16", 4, 28, 4, 128, 65536, 32, POOL_AVG, 5, 1024, 28,
              seed=5, head_key_scale=True, gate=True)
CONFIGS = (C1, C2, C3, C4, C5)

# Length scaling at a fixed retained ratio (the paper's pressure-regime setting: budgets 256 / 512 / 1024 /
# 2048 for 16k / 32k / 64k / 128k contexts) and the extreme 128-token budget at 32k, on C3's attention
# shape. Batch 4 keeps one layer's K and V at 2 GiB for the longest context.
def _sweep(name: str, seq_len: int, budget: int, seed: int) -> Workload:
    return C3.scaled(name=name, batch=4, seq_len=seq_len, budget=budget, seed=seed)


SWEEP = (_sweep("s16k_b256_gqa32x8_bz4", 16384, 256, 11), _sweep("s32k_b512_gqa32x8_bz4", 32768, 512, 12),
         _sweep("s64k_b1024_gqa32x8_bz4", 65536, 1024, 13), _sweep("s128k_b2048_gqa32x8_bz4", 131072, 2048, 14),
         _sweep("s32k_b128_gqa32x8_bz4", 32768, 128, 15))


def _gen(device, *keys: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for k in keys:
        s = (s * 6364136223846793005 + int(k) + 1442695040888963407) % (1 << 63)
    g.manual_seed(s)
    return g


def make_tables(w: Workload, device="cpu") -> dict:
    """Compiled-table stand-ins for every layer: w_head, head_share, t_gate, risk_bins (or None)."""
    g = _gen("cpu", w.seed, 1001)
    w_head = torch.empty(w.n_layers, w.n_q_heads).uniform_(0.5, 1.5, generator=g)
    out = {"w_head": w_head.to(device), "head_share": None, "t_gate": None, "risk_bins": None,
           "n_ent": 0, "n_ppl": 0}
    if w.shares:
        raw = torch.empty(w.n_layers, w.n_kv_heads).uniform_(0.5, 1.5, generator=g)
        out["head_share"] = (raw / raw.sum(dim=1, keepdim=True)).to(device)
    if w.gate:
        n_ent, n_ppl = 20, 4
        level = torch.randint(0, 21, (w.n_layers, n_ent, n_ppl), generator=g)
        out["t_gate"] = (0.8 + 0.01 * level.to(torch.float32)).to(device)
        x = torch.rand(w.batch, 2, generator=g)  # stand-in for the prompt's (entropy, perplexity) risk
        bins = torch.stack([(x[:, 0] * n_ent).long().clamp_(0, n_ent - 1),
                            (x[:, 1] * n_ppl).long().clamp_(0, n_ppl - 1)], dim=1).to(torch.int32)
        out["risk_bins"] = bins.to(device)
        out["n_ent"], out["n_ppl"] = n_ent, n_ppl
    return out


def make_layer(w: Workload, layer: int = 0, device="cpu") -> dict:
    """Q window [Bz,Hq,W,d], K and V [Bz,Hkv,T,d] of one layer in the workload's dtype."""
    Bz, Hq, Hkv, d, T, W = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seq_len, w.window
    dt = w.torch_dtype
    g = _gen(device, w.seed, layer, 1)
    q = torch.randn(Bz, Hq, W, d, generator=g, device=device, dtype=torch.float32).to(dt)
    v = torch.empty(Bz, Hkv, T, d, device=device, dtype=dt)
    k = torch.empty(Bz, Hkv, T, d, device=device, dtype=dt)
    head_scale = None
    if w.head_key_scale:
        u = torch.rand(Bz, Hkv, generator=g, device=device)
        head_scale = torch.exp(math.log(0.5) + u * (math.log(4.0) - math.log(0.5)))
    for b in range(Bz):  # one batch element at a time keeps the fp32 staging buffers small
        kb = torch.randn(Hkv, T, d, generator=g, device=device, dtype=torch.float32)
        if w.pareto_frac > 0:
            hit = torch.rand(Hkv, T, 1, generator=g, device=device) < w.pareto_frac
            u = torch.rand(Hkv, T, 1, generator=g, device=device).clamp_min_(1e-6)
            kb = kb * torch.where(hit, u.rsqrt(), torch.ones_like(u))
        if head_scale is not None:
            kb = kb * head_scale[b].view(Hkv, 1, 1)
        if w.sink_scale:
            kb[:, 0, :] *= w.sink_scale
        k[b] = kb.to(dt)
        v[b] = torch.randn(Hkv, T, d, generator=g, device=device, dtype=torch.float32).to(dt)
        del kb
    needle_pos = None
    if w.needles:
        gc = _gen("cpu", w.seed, layer, 2)
        P, G = w.prefix, w.group
        needle_pos = torch.empty(Bz, Hkv, w.needles, dtype=torch.long)
        for b in range(Bz):
            for kv in range(Hkv):
                lo = 1 if w.sink_scale else 0
                pos = (torch.randperm(P - lo, generator=gc)[: w.needles] + lo).sort().values
                needle_pos[b, kv] = pos
                for n in range(w.needles):
                    h = kv * G + int(torch.randint(0, G, (1,), generator=gc))
                    j = int(torch.randint(0, W, (1,), generator=gc))
                    k[b, kv, pos[n]] = (4.0 * q[b, h, j].to(torch.float32)).to(dt)
    return {"q": q, "k": k, "v": v, "needle_pos": needle_pos}


def make_decode_queries(w: Workload, layer: int, n_q: int, device="cpu") -> torch.Tensor:
    """Queries of n_q decoding steps after the prompt, [Bz,Hq,n_q,d] in the workload's dtype: drawn like
    the window's query rows (the decoding queries of a real model continue the prompt's last rows)."""
    g = _gen(device, w.seed, layer, 2)
    q = torch.randn(w.batch, w.n_q_heads, n_q, w.head_dim, generator=g, device=device, dtype=torch.float32)
    return q.to(w.torch_dtype)
