"""GPU parity at the full sizes of the baseline configurations. Every case runs twice: through the
four separate calls (window scores, tables, selection, gather), and through the call sequence the
benchmark times, in which ckv_window_utility replaces the first two (the per-head window mass is then
never materialised, so the score checks are skipped and the utilities carry the comparison). Layer 0 of
every configuration, a second layer of the benchmark's own workload and the length-scaling rows are
compared with the oracle element by element on every (batch, KV head) unit; on a second layer of the two
largest shapes a seeded unit is compared element by element and every unit is checked through
size-independent properties plus the exact selection / gather stages."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import assert_index_sets_match, assert_scores_close, bits, f32, run_gpu

pytestmark = pytest.mark.gpu
DEV = "cuda"

# (workload, layer, units compared element by element)
ALL = -1  # compare every (batch, KV head) unit with the oracle (it takes the oracle a few seconds per layer)
CASES = [(wl.C2, 0, ALL), (wl.C3, 0, ALL), (wl.C3, 17, ALL), (wl.C4, 0, ALL), (wl.C4, 9, 1), (wl.C5, 0, ALL), (wl.C5, 27, 1)]
# length scaling at the fixed retained ratio 512 / 32k, and the 128-token budget (Sec. 5, pressure regime)
CASES += [(wl.SWEEP[0], 0, ALL), (wl.SWEEP[1], 3, ALL), (wl.SWEEP[2], 0, ALL), (wl.SWEEP[3], 0, ALL), (wl.SWEEP[4], 5, ALL)]


@pytest.mark.parametrize("fused", [False, True], ids=["four_calls", "window_utility"])
@pytest.mark.parametrize("w,layer,n_units", CASES, ids=lambda x: x.name if isinstance(x, wl.Workload) else str(x))
def test_full_size_layer(w, layer, n_units, fused):
    print(f"case {w.name} layer {layer} fused {fused}", flush=True)
    t = wl.make_layer(w, layer, DEV)
    tabs = wl.make_tables(w, DEV)
    p, buf = run_gpu(w, t, tabs, layer=layer, fused_utility=fused)
    Bz, Hq, Hkv, G, T, W, P = w.batch, w.n_q_heads, w.n_kv_heads, w.group, w.seq_len, w.window, w.prefix

    # ---- properties that hold at any size, over every unit -------------------------------------
    if not fused:
        s = buf.scores
        assert torch.isfinite(s).all() and (s >= 0).all()
        np.testing.assert_allclose(s.double().sum(-1).cpu().numpy(), T, rtol=2e-4)      # Eq. 4 remark
    assert torch.isfinite(buf.utility).all() and (buf.utility >= 0).all()
    budget, count, tau = buf.budget.cpu().numpy(), buf.count.cpu().numpy(), buf.tau.cpu().numpy()
    assert (budget >= W).all() and (budget <= min(T, w.cap)).all()
    assert (budget.sum(1) <= w.budget * Hkv).all()
    share = tabs["head_share"]
    ref_b = oracle.budgets(Hkv, T, W, w.budget, None if share is None else f32(share[layer]))
    np.testing.assert_array_equal(budget, np.tile(ref_b, (Bz, 1)))
    if tabs["t_gate"] is not None:
        bins = tabs["risk_bins"].cpu().numpy()
        ref_tau = [oracle.tau(f32(tabs["t_gate"][layer]), bins[b, 0], bins[b, 1]) for b in range(Bz)]
        np.testing.assert_array_equal(tau, np.array(ref_tau, np.float32))
    else:
        assert (tau == 0).all()
    ncand = (buf.utility >= buf.tau[:, None, None]).sum(-1).cpu().numpy()
    np.testing.assert_array_equal(count, np.minimum(budget, W + ncand))                 # clamped budget
    if w.budget * 64 == T:
        np.testing.assert_allclose(count.sum(1) / (Hkv * T), 0.015625, atol=1e-4)        # Table A6: 1.56 %

    # ---- selection and gather: exact, every unit, from the GPU's own utilities ------------------
    util = buf.utility.cpu().numpy()
    gi, gc = buf.idx.cpu().numpy(), count
    oi, oc = oracle.select(util, tau, budget, W, w.cap)
    np.testing.assert_array_equal(gc, oc)
    np.testing.assert_array_equal(gi, oi)
    for b in range(Bz):
        for g in range(Hkv):
            c = gc[b, g]
            assert gi[b, g, c - W:c].tolist() == list(range(P, T))                        # window kept, last
    kb, vb = bits(t["k"]), bits(t["v"])
    np.testing.assert_array_equal(bits(buf.k_out), oracle.gather(kb, gi, gc))
    np.testing.assert_array_equal(bits(buf.v_out), oracle.gather(vb, gi, gc))
    del kb, vb
    if t["needle_pos"] is not None:
        for b in range(Bz):
            for g in range(Hkv):
                assert set(t["needle_pos"][b, g].tolist()) <= set(gi[b, g, : gc[b, g]].tolist())

    # ---- every unit against the oracle, element by element (n_units = ALL) -------------------------
    if n_units == ALL:
        ref_s = oracle.window_scores(f32(t["q"]), f32(t["k"]))          # all (batch, head) units at once
        if not fused:
            assert_scores_close(buf.scores.cpu().numpy(), ref_s, "scores, every unit")
        ref_u = oracle.utility(ref_s, W, Hkv, w.pool, w.pool_kernel, f32(tabs["w_head"][layer]))
        del ref_s
        assert_scores_close(util, ref_u.astype(np.float64), "utility, every unit")
        ri, rc = oracle.select(ref_u, tau, budget, W, w.cap)
        assert_index_sets_match(gi, gc, ri, rc, ref_u, tau, budget, W)
        return

    # ---- sampled units against the oracle, element by element ------------------------------------
    rng = np.random.default_rng(w.seed * 1000 + layer)
    for u in sorted(rng.choice(Bz * Hkv, size=max(n_units, 1), replace=False).tolist()):
        b, g = divmod(u, Hkv)
        print(f"  unit (b={b}, g={g})", flush=True)
        q_u = f32(t["q"][b:b + 1, g * G:(g + 1) * G])
        k_u = f32(t["k"][b:b + 1, g:g + 1])
        ref_s = oracle.window_scores(q_u, k_u)
        if not fused:
            assert_scores_close(buf.scores[b, g * G:(g + 1) * G].cpu().numpy()[None], ref_s, f"scores unit {u}")
        w_row = f32(tabs["w_head"][layer])[g * G:(g + 1) * G]
        ref_u = oracle.utility(ref_s, W, 1, w.pool, w.pool_kernel, w_row)
        assert_scores_close(util[b:b + 1, g:g + 1], ref_u.astype(np.float64), f"utility unit {u}")
        ri, rc = oracle.select(ref_u, tau[b:b + 1], budget[b:b + 1, g:g + 1], W, w.cap)
        assert_index_sets_match(gi[b:b + 1, g:g + 1], gc[b:b + 1, g:g + 1], ri, rc, ref_u, tau[b:b + 1],
                                budget[b:b + 1, g:g + 1], W)
