"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI, run the oracle on
host copies of the same tensors, and the comparison rules."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl

SCORE_RTOL = 1e-3      # fp32 scores: |gpu - ref| <= 1e-3 * max(|ref|, 1e-6)
SCORE_FLOOR = 1e-6
GAP = 1e-4             # index sets must match exactly wherever the boundary gap exceeds this


def f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float32).contiguous().numpy()


def bits(t: torch.Tensor) -> np.ndarray:
    t = t.detach().to("cpu").contiguous()
    return t.view(torch.int16).numpy() if t.dtype == torch.bfloat16 else t.numpy()


def params_of(w: wl.Workload, q, k, v, layer=0, flags=0, cap=None) -> B.CkvParams:
    return B.params_for(q, k, v, pool=w.pool, pool_kernel=w.pool_kernel, budget=w.budget,
                        cap=w.cap if cap is None else cap, layer=layer, n_layers=w.n_layers, flags=flags)


def run_gpu(w: wl.Workload, layer_t: dict, tables: dict, layer=0, flags=0, lse=None, fused_utility=False):
    """fused_utility: ckv_window_utility in place of ckv_window_scores + ckv_apply_tables (what bench.py
    times); buf.scores is then scratch, prefilled with NaN like buf.utility so that a position the
    kernels leave unwritten shows up."""
    q, k, v = layer_t["q"], layer_t["k"], layer_t["v"]
    p = params_of(w, q, k, v, layer, flags)
    buf = B.LayerBuffers(p, q.device)
    if fused_utility:
        buf.scores.fill_(float("nan"))
        buf.utility.fill_(float("nan"))
    B.retention_layer(p, q, k, v, tables, buf, lse=lse, fused_utility=fused_utility)
    torch.cuda.synchronize()
    return p, buf


def run_oracle(w: wl.Workload, layer_t: dict, tables: dict, layer=0, value_norm=False):
    q, k, v = layer_t["q"], layer_t["k"], layer_t["v"]
    share = tables["head_share"]
    gate = tables["t_gate"]
    return oracle.retention_layer(
        f32(q), f32(k), bits(v), v=f32(v) if value_norm else None, W=w.window, mode=w.pool,
        kernel=w.pool_kernel, B=w.budget, cap=w.cap, w_head_row=f32(tables["w_head"][layer]),
        share_row=None if share is None else f32(share[layer]),
        gate_layer=None if gate is None else f32(gate[layer]),
        risk_bins=None if gate is None else tables["risk_bins"].cpu().tolist(),
        value_norm=value_norm, k_bits=bits(k))


def assert_scores_close(gpu: np.ndarray, ref: np.ndarray, what="scores"):
    gpu = np.asarray(gpu, dtype=np.float64)
    err = np.abs(gpu - ref)
    tol = SCORE_RTOL * np.maximum(np.abs(ref), SCORE_FLOOR)
    bad = err > tol
    assert np.isfinite(gpu).all(), f"{what}: non-finite values"
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst rel err "
                           f"{(err / np.maximum(np.abs(ref), SCORE_FLOOR)).max():.3e} at {np.argwhere(bad)[:3].tolist()}")


def assert_index_sets_match(gpu_idx, gpu_count, ref_idx, ref_count, ref_utility, tau, budget, W):
    """Exact match per unit, unless the oracle's own boundary is closer than GAP: then the symmetric
    difference must lie inside the +-GAP band around the boundary value (k-th utility or tau)."""
    Bz, Hkv, P = ref_utility.shape
    n_loose = 0
    for b in range(Bz):
        for g in range(Hkv):
            cg, cr = int(gpu_count[b, g]), int(ref_count[b, g])
            ig, ir = gpu_idx[b, g, :cg], ref_idx[b, g, :cr]
            if cg == cr and np.array_equal(ig, ir):
                continue
            u = ref_utility[b, g].astype(np.float64)
            kp = int(budget[b, g]) - W
            cand = u[u >= tau[b]]
            # the gate's threshold is a boundary only where it can exclude something (tau = 0: gate off)
            bounds = [float(tau[b])] if tau[b] > 0 else []
            if len(cand) > kp > 0:
                srt = np.sort(cand)[::-1]
                bounds.append(float(srt[kp - 1]))
            diff = np.setxor1d(ig[: cg - W], ir[: cr - W])
            near = np.zeros(len(diff), dtype=bool)
            for bd in bounds:
                near |= np.abs(u[diff] - bd) <= GAP
            assert near.all(), (f"unit ({b},{g}): index sets differ outside the {GAP} band: "
                                f"{diff[~near][:5].tolist()} utilities {u[diff[~near]][:5]}")
            assert np.array_equal(ig[cg - W:], ir[cr - W:]), "window tail differs"
            n_loose += 1
    return n_loose
