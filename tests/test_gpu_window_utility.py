"""GPU parity of ckv_window_utility (scan + tables in one call, the per-head window mass not
materialised): against the CPU oracle, and against the two unfused calls on the same tensors.

The fused second pass works on 128-key pipeline rounds per wave: the first and the last round of a
wave's key range treat their edges specially (raw column sums for the fix-up kernel), rounds in between
only carry the previous round's tail in front. The shapes marked "rounds" give every wave at least
three rounds (batch x KV heads x T >= 3 * 128 * 1024 keys over the 1024 waves of a launch), so that
first, middle and last rounds all meet the oracle, for every pooling mode and radius the fused pass
takes and for both head sizes. wu_short has no whole round at all (range tails and the fix-up kernel
only). The last group holds shapes the fused pass does not take: they run the two steps through the
scratch buffer."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import assert_index_sets_match, assert_scores_close, bits, f32, params_of, run_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(name, dtype, Bz, Hq, Hkv, d, T, W, pool, kernel, budget, **kw):
    return wl.Workload(name, dtype, Bz, Hq, Hkv, d, T, W, pool, kernel, budget, 2, seed=500 + T + W + Hq + kernel, **kw)


# (workload, value norm)
CASES = [
    # rounds per wave >= 3 (first, middle and last rounds of the fused flush)
    (_case("wu_gqa4_avg7", "bf16", 4, 8, 2, 128, 49152, 32, wl.POOL_AVG, 7, 600, shares=True, pareto_frac=0.05), False),
    (_case("wu_gqa4_max7_ragged", "bf16", 4, 8, 2, 128, 50004, 32, wl.POOL_MAX, 7, 700, needles=5, sink_scale=8.0), False),
    (_case("wu_mha_avg5_gate", "bf16", 6, 2, 2, 128, 36000, 32, wl.POOL_AVG, 5, 300, gate=True), False),
    (_case("wu_gqa3_max3", "bf16", 3, 6, 2, 128, 66000, 32, wl.POOL_MAX, 3, 500, head_key_scale=True), False),
    (_case("wu_gqa2_avg3", "bf16", 4, 4, 2, 128, 50000, 32, wl.POOL_AVG, 3, 400, shares=True), False),
    (_case("wu_gqa4_max5", "bf16", 2, 16, 4, 128, 50000, 32, wl.POOL_MAX, 5, 300), False),
    (_case("wu_gqa2_nopool_w20", "bf16", 6, 4, 2, 128, 33000, 20, wl.POOL_NONE, 1, 400, shares=True), False),
    (_case("wu_d64_avg7", "bf16", 2, 16, 4, 64, 70000, 32, wl.POOL_AVG, 7, 400), False),
    (_case("wu_d64_max3", "bf16", 2, 8, 4, 64, 52000, 32, wl.POOL_MAX, 3, 300), False),
    (_case("wu_value_norm_rounds", "bf16", 2, 8, 4, 128, 50000, 32, wl.POOL_AVG, 7, 300), True),
    # five to eight query tiles per wave, and two tiles per head (W = 64)
    (_case("wu_gqa7_avg5", "bf16", 2, 14, 2, 128, 66000, 32, wl.POOL_AVG, 5, 600, head_key_scale=True, gate=True), False),
    (_case("wu_gqa8_max7", "bf16", 1, 16, 2, 128, 140000, 32, wl.POOL_MAX, 7, 500, needles=4), False),
    (_case("wu_gqa5_avg3_d64", "bf16", 2, 10, 2, 64, 100000, 32, wl.POOL_AVG, 3, 400), False),
    (_case("wu_gqa6_nopool", "bf16", 4, 6, 1, 128, 100000, 24, wl.POOL_NONE, 1, 300), False),
    (_case("wu_gqa4_w64_max7", "bf16", 1, 8, 2, 128, 200000, 64, wl.POOL_MAX, 7, 700, needles=6, sink_scale=8.0, shares=True), False),
    (_case("wu_gqa3_w48_avg7", "bf16", 2, 6, 2, 128, 100000, 48, wl.POOL_AVG, 7, 500), False),
    (_case("wu_gqa2_w64_avg5_d64", "bf16", 2, 4, 2, 64, 100000, 64, wl.POOL_AVG, 5, 400, shares=True), False),
    (_case("wu_gqa4_w64_value_norm", "bf16", 4, 8, 2, 128, 50000, 64, wl.POOL_AVG, 7, 300), True),
    # fewer rounds, and none at all
    (_case("wu_gqa3_two_rounds", "bf16", 1, 6, 2, 128, 100000, 32, wl.POOL_AVG, 5, 500), False),
    (_case("wu_short", "bf16", 2, 8, 2, 128, 1000, 32, wl.POOL_AVG, 7, 200), False),           # tails only
    (_case("wu_value_norm", "bf16", 1, 8, 2, 128, 20000, 32, wl.POOL_AVG, 7, 300), True),
    (_case("wu_value_norm_max_gqa3", "bf16", 2, 6, 2, 128, 9000, 32, wl.POOL_MAX, 5, 200), True),
    # shapes the fused pass does not take: they run the two steps through the scratch buffer
    (_case("wu_avg9", "bf16", 1, 8, 2, 128, 20000, 32, wl.POOL_AVG, 9, 300), False),            # radius 4
    (_case("wu_w96", "bf16", 1, 4, 2, 128, 20000, 96, wl.POOL_MAX, 7, 300), False),             # three tiles per head
    (_case("wu_odd_prefix", "bf16", 1, 4, 2, 128, 20000, 30, wl.POOL_AVG, 7, 300), False),      # P % 4 != 0
    (_case("wu_f32", "f32", 1, 4, 4, 64, 2048, 32, wl.POOL_AVG, 7, 200, shares=True), False),
]


@pytest.mark.parametrize("w,vn", CASES, ids=lambda x: x.name if isinstance(x, wl.Workload) else f"vn{int(x)}")
def test_window_utility_matches_oracle_and_unfused(w, vn):
    print(f"case {w.name}", flush=True)
    layer, tabs = wl.make_layer(w, 1, DEV), wl.make_tables(w, DEV)
    q, k, v = layer["q"], layer["k"], layer["v"]
    p = params_of(w, q, k, v, layer=1, flags=B.FLAG_VALUE_NORM if vn else 0)
    fused, plain = B.LayerBuffers(p, DEV), B.LayerBuffers(p, DEV)
    for buf in (fused, plain):
        buf.utility.fill_(float("nan"))
        buf.scores.fill_(float("nan"))
    B.retention_layer(p, q, k, v, tabs, fused, fused_utility=True)
    B.retention_layer(p, q, k, v, tabs, plain)
    torch.cuda.synchronize()
    ref = run_oracle(w, layer, tabs, layer=1, value_norm=vn)
    fu, pu = fused.utility.cpu().numpy(), plain.utility.cpu().numpy()
    assert_scores_close(fu, ref["utility"].astype(np.float64), "fused utility")
    # same column sums, same taps in the same order; only the division by the kernel size is a
    # multiplication by its reciprocal in the fused pass
    # (with the value norm the fused pass multiplies the group maximum by rho, the unfused one each head's
    # term: one rounding more on either side)
    np.testing.assert_allclose(fu, pu, rtol=1e-6 if vn else 3e-7, atol=0)
    if vn:
        assert_scores_close(fused.vnorm_ratio.cpu().numpy(), ref["rho"], "rho")
        np.testing.assert_array_equal(fused.vnorm_ratio.cpu().numpy(), plain.vnorm_ratio.cpu().numpy())
    np.testing.assert_array_equal(fused.budget.cpu().numpy(), ref["budget"])
    np.testing.assert_array_equal(fused.tau.cpu().numpy(), ref["tau"])
    gi, gc = fused.idx.cpu().numpy(), fused.count.cpu().numpy()
    assert_index_sets_match(gi, gc, ref["idx"], ref["count"], ref["utility"], ref["tau"], ref["budget"], w.window)
    oi, oc = oracle.select(fu, fused.tau.cpu().numpy(), fused.budget.cpu().numpy(), w.window, w.cap)
    np.testing.assert_array_equal(gc, oc)
    np.testing.assert_array_equal(gi, oi)
    np.testing.assert_array_equal(bits(fused.k_out), oracle.gather(bits(k), gi, gc))
    np.testing.assert_array_equal(bits(fused.v_out), oracle.gather(bits(v), gi, gc))


def test_window_utility_full_size_c3_layer():
    """The benchmark's launch configuration: every unit against the unfused calls, properties on all."""
    w = wl.C3
    t, tabs = wl.make_layer(w, 5, DEV), wl.make_tables(w, DEV)
    q, k, v = t["q"], t["k"], t["v"]
    p = params_of(w, q, k, v, layer=5)
    fused, plain = B.LayerBuffers(p, DEV), B.LayerBuffers(p, DEV)
    fused.utility.fill_(float("nan"))
    B.retention_layer(p, q, k, v, tabs, fused, fused_utility=True)
    B.retention_layer(p, q, k, v, tabs, plain)
    torch.cuda.synchronize()
    assert torch.isfinite(fused.utility).all()
    np.testing.assert_allclose(fused.utility.cpu().numpy(), plain.utility.cpu().numpy(), rtol=3e-7, atol=0)
    assert torch.equal(fused.budget, plain.budget) and torch.equal(fused.tau, plain.tau)
    fu = fused.utility.cpu().numpy()
    oi, oc = oracle.select(fu, fused.tau.cpu().numpy(), fused.budget.cpu().numpy(), w.window, w.cap)
    np.testing.assert_array_equal(fused.count.cpu().numpy(), oc)
    np.testing.assert_array_equal(fused.idx.cpu().numpy(), oi)
    np.testing.assert_allclose(oc.sum(1) / (w.n_kv_heads * w.seq_len), 0.015625, atol=1e-4)   # Table A6: 1.56 %
    # one unit against the oracle, element by element
    b, g, G = 7, 3, w.group
    ref_s = oracle.window_scores(f32(q[b:b + 1, g * G:(g + 1) * G]), f32(k[b:b + 1, g:g + 1]))
    ref_u = oracle.utility(ref_s, w.window, 1, w.pool, w.pool_kernel, f32(tabs["w_head"][5])[g * G:(g + 1) * G])
    assert_scores_close(fu[b:b + 1, g:g + 1], ref_u.astype(np.float64), "utility of unit (7, 3)")
