"""Seeded sweep over shapes nobody picked by hand: element type, head size, group size, window (1..128,
ragged), length (ragged, up to 120k, bounded so that the oracle takes seconds), pooling mode and kernel, value
norm, gate, shares, batch. Every shape runs the whole chain through the C ABI both ways (the four separate
calls; ckv_window_utility in place of the first two, which falls back to the two steps where its fused
pass does not apply) and, for half of them, with the oracle's LSE handed in; each run is compared with the
oracle like the hand-picked chain cases: scores / utilities element by element, budgets and thresholds
exactly, index sets exactly outside the tolerance band, selection and gather bit for bit from the GPU's own
utilities."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import assert_index_sets_match, assert_scores_close, bits, f32, params_of, run_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda"
# the committed sweep; CKV_RANDOM_SHAPES="<first seed>:<count>" draws another one
FIRST_SEED, N_SHAPES = (int(x) for x in os.environ.get("CKV_RANDOM_SHAPES", "9000:48").split(":"))


def _draw(i: int):
    rng = np.random.default_rng(FIRST_SEED + i)
    dtype = "f32" if rng.random() < 0.25 else "bf16"
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.integers(1, 5 if dtype == "f32" else 9))
    W = int(rng.choice([1, 7, 16, 20, 32, 32, 32, 33, 48, 64, 64, 96, 128]))
    # lengths from a few tiles to several pipeline rounds per wave; every residue modulo 32 and 4 occurs
    t_max = min(120000.0, 6e9 / (G * Hkv * W * d))   # bounds the oracle's time per case to a few seconds
    T = W + int(rng.integers(0, 3)) * int(rng.integers(0, 40)) + int(np.exp(rng.uniform(np.log(40), np.log(t_max))))
    pool = int(rng.choice([wl.POOL_NONE, wl.POOL_AVG, wl.POOL_MAX]))
    kernel = 1 if pool == wl.POOL_NONE else int(rng.choice([1, 3, 5, 7, 7, 9, 15]))
    Bz = int(rng.integers(1, 3))
    budget = W + int(rng.integers(0, max(1, (T - W) // 3) + 1))
    kw = dict(shares=bool(rng.random() < 0.5), gate=bool(rng.random() < 0.4))
    if rng.random() < 0.3:
        kw["pareto_frac"] = 0.05
    if rng.random() < 0.3:
        kw["sink_scale"] = 8.0
    if rng.random() < 0.3:
        kw["head_key_scale"] = True
    w = wl.Workload(f"rnd{i}_{dtype}_g{G}x{Hkv}_d{d}_T{T}_W{W}_p{pool}k{kernel}", dtype, Bz, G * Hkv, Hkv, d, T, W, pool,
                    kernel, budget, 3, seed=FIRST_SEED - 2000 + i, **kw)
    return w, bool(rng.random() < 0.35), bool(rng.random() < 0.5), int(rng.integers(0, 3))


CASES = [_draw(i) for i in range(N_SHAPES)]


@pytest.mark.parametrize("w,vn,given_lse,layer", CASES, ids=lambda x: x.name if isinstance(x, wl.Workload) else str(int(x)))
def test_random_shape_chain_matches_oracle(w, vn, given_lse, layer):
    print(f"case {w.name} value_norm={vn} given_lse={given_lse} layer={layer}", flush=True)
    t, tabs = wl.make_layer(w, layer, DEV), wl.make_tables(w, DEV)
    q, k, v = t["q"], t["k"], t["v"]
    ref = run_oracle(w, t, tabs, layer=layer, value_norm=vn)
    lse = None
    if given_lse:
        _, lse_ref = oracle.window_scores(f32(q), f32(k), return_lse=True)
        lse = torch.from_numpy(lse_ref.astype(np.float32)).to(DEV)
    p = params_of(w, q, k, v, layer=layer, flags=B.FLAG_VALUE_NORM if vn else 0)
    for fused in (False, True):
        buf = B.LayerBuffers(p, DEV)
        buf.scores.fill_(float("nan"))
        buf.utility.fill_(float("nan"))
        B.retention_layer(p, q, k, v, tabs, buf, lse=lse, fused_utility=fused)
        torch.cuda.synchronize()
        what = "window_utility" if fused else "four calls"
        if not fused:
            assert_scores_close(buf.scores.cpu().numpy(), ref["scores"], f"scores ({what})")
        if vn:
            assert_scores_close(buf.vnorm_ratio.cpu().numpy(), ref["rho"], f"rho ({what})")
        gu = buf.utility.cpu().numpy()
        assert_scores_close(gu, ref["utility"].astype(np.float64), f"utility ({what})")
        np.testing.assert_array_equal(buf.budget.cpu().numpy(), ref["budget"])
        np.testing.assert_array_equal(buf.tau.cpu().numpy(), ref["tau"])
        gi, gc = buf.idx.cpu().numpy(), buf.count.cpu().numpy()
        assert_index_sets_match(gi, gc, ref["idx"], ref["count"], ref["utility"], ref["tau"], ref["budget"], w.window)
        oi, oc = oracle.select(gu, buf.tau.cpu().numpy(), buf.budget.cpu().numpy(), w.window, w.cap)
        np.testing.assert_array_equal(gc, oc)
        np.testing.assert_array_equal(gi, oi)
        np.testing.assert_array_equal(bits(buf.k_out), oracle.gather(bits(k), gi, gc))
        np.testing.assert_array_equal(bits(buf.v_out), oracle.gather(bits(v), gi, gc))
