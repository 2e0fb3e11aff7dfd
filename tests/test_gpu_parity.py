"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same tensors.

Small cases compare every element; the full-size cases run the launch configuration the benchmark
times and compare sampled (batch, KV head) units element by element plus size-independent
properties on everything.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import (assert_index_sets_match, assert_scores_close, bits, f32, params_of, run_gpu,
                         run_oracle)

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _small(name, dtype, Bz, Hq, Hkv, d, T, W, pool=wl.POOL_AVG, kernel=7, B_=None, **kw):
    B_ = B_ if B_ is not None else max(W + 8, min(T, W + T // 8))
    return wl.Workload(name, dtype, Bz, Hq, Hkv, d, T, W, pool, kernel, B_, 2, seed=100 + T + W + Hq, **kw)


SCORE_CASES = [
    _small("f32_mha", "f32", 1, 4, 4, 64, 1024, 32),
    _small("f32_gqa_ragged", "f32", 2, 6, 2, 64, 777, 20),          # ragged tail, ragged window, NQ=3
    _small("f32_d128", "f32", 1, 2, 1, 128, 300, 32),
    _small("bf16_mha", "bf16", 1, 8, 8, 128, 2048, 32, sink_scale=8.0),
    _small("bf16_gqa4", "bf16", 2, 8, 2, 128, 4133, 32, pareto_frac=0.05),   # NQ=4, ragged tail
    _small("bf16_gqa4_w64", "bf16", 1, 8, 2, 128, 3000, 64, needles=4),      # two tiles per head
    _small("bf16_gqa7", "bf16", 1, 7, 1, 128, 2500, 32, head_key_scale=True),  # seven tiles in one wave
    _small("bf16_gqa5_w48", "bf16", 1, 5, 1, 128, 1500, 48),                 # WT=2, padded rows, groups of 6 + 4 tiles
    _small("bf16_gqa5", "bf16", 2, 10, 2, 128, 1700, 32),                    # five tiles per wave
    _small("bf16_gqa6_d64", "bf16", 1, 6, 1, 64, 2100, 32),                  # six tiles, 128-byte rows
    _small("bf16_gqa8", "bf16", 1, 16, 2, 128, 1900, 32, sink_scale=8.0),    # eight tiles, one per head
    _small("bf16_gqa12", "bf16", 1, 12, 1, 128, 1300, 32),                   # two groups of six tiles
    _small("bf16_gqa2_w96", "bf16", 1, 4, 2, 128, 1400, 96, B_=200),         # three tiles per head, six per wave
    _small("bf16_gqa2_w128_d64", "bf16", 1, 2, 1, 64, 1200, 128, B_=200),    # four tiles per head, eight per wave
    _small("bf16_d64", "bf16", 1, 4, 2, 64, 1111, 32),
    _small("bf16_w1", "bf16", 1, 2, 2, 128, 500, 1),
    _small("bf16_all_window", "bf16", 1, 2, 1, 128, 32, 32, B_=32),         # P = 0
    _small("bf16_tiny", "bf16", 1, 1, 1, 128, 40, 8),
    _small("bf16_w128", "bf16", 1, 2, 2, 128, 1000, 128, B_=200),
]


@pytest.mark.parametrize("w", SCORE_CASES, ids=lambda w: w.name)
def test_window_scores_match_oracle(w):
    print(f"case {w.name}", flush=True)
    layer = wl.make_layer(w, 0, DEV)
    q, k, v = layer["q"], layer["k"], layer["v"]
    p = params_of(w, q, k, v)
    buf = B.LayerBuffers(p, DEV)
    buf.scores.fill_(float("nan"))
    B.ckv_window_scores(p, q, k, None, None, buf.scores, None, buf.workspace)
    torch.cuda.synchronize()
    ref, lse = oracle.window_scores(f32(q), f32(k), return_lse=True)
    got = buf.scores.cpu().numpy()
    assert_scores_close(got, ref)
    np.testing.assert_allclose(got.astype(np.float64).sum(-1), w.seq_len, rtol=2e-4)   # Eq. 4 remark
    # caller-supplied LSE: single pass over K, same result
    lse_t = torch.from_numpy(lse.astype(np.float32)).to(DEV)
    buf.scores.fill_(float("nan"))
    B.ckv_window_scores(p, q, k, None, lse_t, buf.scores, None, buf.workspace)
    torch.cuda.synchronize()
    assert_scores_close(buf.scores.cpu().numpy(), ref, "scores with given LSE")


# Long enough, with few enough (batch, KV head) units, that every wave's key range spans whole rounds of
# the scan kernels' four-tile software pipeline (the cases above mostly take its masked tail path):
# odd group sizes, several tiles per head, 128-byte rows, ragged ends.
PIPELINE_CASES = [
    _small("long_gqa7", "bf16", 1, 7, 1, 128, 70001, 32, pareto_frac=0.05),       # seven tiles per wave
    _small("long_gqa5", "bf16", 1, 5, 1, 128, 90001, 32),                         # five tiles per wave
    _small("long_gqa6_d64", "bf16", 1, 6, 1, 64, 80002, 32),                      # six tiles, 128-byte rows
    _small("long_gqa8", "bf16", 1, 8, 1, 128, 70003, 32, sink_scale=8.0),         # eight tiles, one per head
    _small("long_gqa3_w64", "bf16", 1, 3, 1, 128, 60000, 64),                     # six tiles, two per head
    _small("long_gqa2_w96", "bf16", 1, 2, 1, 128, 60001, 96, B_=300),             # six tiles, three per head
    _small("long_gqa2_w128", "bf16", 1, 4, 2, 128, 50000, 128, B_=300),           # eight tiles, four per head
    _small("long_gqa9", "bf16", 1, 9, 1, 128, 40000, 32),                         # two groups: 5 + 4 tiles
    _small("long_gqa3", "bf16", 1, 3, 1, 128, 140003, 32, sink_scale=8.0),        # three tiles per wave
    _small("long_w64", "bf16", 1, 8, 2, 128, 40000, 64, needles=4),               # two tiles per head
    _small("long_w128", "bf16", 1, 2, 2, 128, 70000, 128, B_=300),                # four tiles per head
    _small("long_w48_gqa5", "bf16", 1, 5, 1, 128, 50000, 48),                     # padded second tile, groups of 3 + 2 heads
    _small("long_d64", "bf16", 1, 4, 2, 64, 70003, 32, head_key_scale=True),      # 128-byte rows
    _small("long_mha", "bf16", 1, 2, 2, 128, 66000, 32),                          # one tile per wave
]


@pytest.mark.parametrize("w", PIPELINE_CASES, ids=lambda w: w.name)
def test_window_scores_pipelined_shapes(w):
    print(f"case {w.name}", flush=True)
    layer = wl.make_layer(w, 0, DEV)
    q, k, v = layer["q"], layer["k"], layer["v"]
    p = params_of(w, q, k, v)
    buf = B.LayerBuffers(p, DEV)
    buf.scores.fill_(float("nan"))
    B.ckv_window_scores(p, q, k, None, None, buf.scores, None, buf.workspace)
    torch.cuda.synchronize()
    ref = oracle.window_scores(f32(q), f32(k))
    got = buf.scores.cpu().numpy()
    assert_scores_close(got, ref)
    np.testing.assert_allclose(got.astype(np.float64).sum(-1), w.seq_len, rtol=2e-4)


def test_window_scores_strided_inputs():
    # K/V as slices of a fused [Bz, T, Hkv, 2, d] cache, Q as a slice of a longer query tensor
    w = _small("strided", "bf16", 2, 8, 2, 128, 1000, 32)
    layer = wl.make_layer(w, 0, DEV)
    kv = torch.empty(w.batch, w.seq_len, w.n_kv_heads, 2, w.head_dim, dtype=torch.bfloat16, device=DEV)
    kv[:, :, :, 0] = layer["k"].transpose(1, 2)
    kv[:, :, :, 1] = layer["v"].transpose(1, 2)
    k, v = kv[:, :, :, 0].transpose(1, 2), kv[:, :, :, 1].transpose(1, 2)
    qfull = torch.zeros(w.batch, w.n_q_heads, 50, w.head_dim, dtype=torch.bfloat16, device=DEV)
    qfull[:, :, 18:] = layer["q"]
    q = qfull[:, :, 18:]
    assert not k.is_contiguous() and not q.is_contiguous()
    tabs = wl.make_tables(w, DEV)
    p = params_of(w, q, k, v, flags=B.FLAG_VALUE_NORM)
    buf = B.LayerBuffers(p, DEV)
    B.retention_layer(p, q, k, v, tabs, buf)
    torch.cuda.synchronize()
    ref = run_oracle(w, layer, tabs, value_norm=True)
    assert_scores_close(buf.scores.cpu().numpy(), ref["scores"])
    assert_scores_close(buf.vnorm_ratio.cpu().numpy(), ref["rho"], "rho")
    n = assert_index_sets_match(buf.idx.cpu().numpy(), buf.count.cpu().numpy(), ref["idx"], ref["count"],
                                ref["utility"], ref["tau"], ref["budget"], w.window)
    if n == 0:
        np.testing.assert_array_equal(bits(buf.k_out), ref["k_out"])
        np.testing.assert_array_equal(bits(buf.v_out), ref["v_out"])


CHAIN_CASES = [
    (wl.C1, False),
    (wl.C1, True),
    (_small("chain_bf16_gqa_gate", "bf16", 3, 8, 2, 128, 3001, 32, wl.POOL_AVG, 5, 200, gate=True,
            head_key_scale=True), False),
    (_small("chain_bf16_max_shares", "bf16", 2, 12, 4, 128, 2222, 64, wl.POOL_MAX, 7, 300, shares=True,
            needles=5, sink_scale=8.0), True),
    (_small("chain_f32_nopool", "f32", 1, 4, 2, 64, 900, 16, wl.POOL_NONE, 1, 100, shares=True), False),
    (_small("chain_long_gqa7", "bf16", 1, 7, 1, 128, 60004, 32, wl.POOL_AVG, 7, 600, gate=True, needles=6), True),
]


@pytest.mark.parametrize("w,vn", CHAIN_CASES, ids=lambda x: x.name if isinstance(x, wl.Workload) else f"vn{int(x)}")
def test_chain_matches_oracle(w, vn):
    print(f"case {w.name} value_norm={vn}", flush=True)
    layer, tabs = wl.make_layer(w, 1 % w.n_layers, DEV), wl.make_tables(w, DEV)
    lay = 1 % w.n_layers
    flags = B.FLAG_VALUE_NORM if vn else 0
    p, buf = run_gpu(w, layer, tabs, layer=lay, flags=flags)
    ref = run_oracle(w, layer, tabs, layer=lay, value_norm=vn)
    assert_scores_close(buf.scores.cpu().numpy(), ref["scores"])
    if vn:
        assert_scores_close(buf.vnorm_ratio.cpu().numpy(), ref["rho"], "rho")
    assert_scores_close(buf.utility.cpu().numpy(), ref["utility"].astype(np.float64), "utility")
    np.testing.assert_array_equal(buf.budget.cpu().numpy(), ref["budget"])
    np.testing.assert_array_equal(buf.tau.cpu().numpy(), ref["tau"])
    gi, gc = buf.idx.cpu().numpy(), buf.count.cpu().numpy()
    n_loose = assert_index_sets_match(gi, gc, ref["idx"], ref["count"], ref["utility"], ref["tau"],
                                      ref["budget"], w.window)
    # Stage-exact checks on the GPU's own intermediates: same utility in => same indices out, bit for bit
    oi, oc = oracle.select(buf.utility.cpu().numpy(), buf.tau.cpu().numpy(), buf.budget.cpu().numpy(),
                           w.window, w.cap)
    np.testing.assert_array_equal(gc, oc)
    np.testing.assert_array_equal(gi, oi)
    np.testing.assert_array_equal(bits(buf.k_out), oracle.gather(bits(layer["k"]), gi, gc))
    np.testing.assert_array_equal(bits(buf.v_out), oracle.gather(bits(layer["v"]), gi, gc))
    if n_loose == 0:
        np.testing.assert_array_equal(bits(buf.k_out), ref["k_out"])
    if layer["needle_pos"] is not None:
        for b in range(w.batch):
            for g in range(w.n_kv_heads):
                kept = set(gi[b, g, : gc[b, g]].tolist())
                assert set(layer["needle_pos"][b, g].tolist()) <= kept


def test_apply_tables_from_identical_scores():
    # Feed the oracle's scores (rounded to fp32) to the GPU stage and the same fp32 values to the oracle.
    rng = np.random.default_rng(5)
    for (Hq, Hkv, T, W, pool, kernel, vn) in [(8, 2, 5000, 32, wl.POOL_AVG, 7, True),
                                               (6, 6, 1025, 16, wl.POOL_MAX, 5, False),
                                               (4, 1, 2048 + 32, 32, wl.POOL_AVG, 63, False),
                                               (4, 2, 700, 64, wl.POOL_NONE, 1, True)]:
        Bz, n_layers = 2, 3
        s = (rng.random((Bz, Hq, T)) ** 4 * 5).astype(np.float32)
        rho = (rng.random((Bz, Hkv, T)) + 0.5).astype(np.float32)
        w_head = (rng.random((n_layers, Hq)) + 0.5).astype(np.float32)
        share = rng.random((n_layers, Hkv)).astype(np.float32)
        share /= share.sum(1, keepdims=True)
        gate = (0.8 + 0.01 * rng.integers(0, 21, (n_layers, 20, 4))).astype(np.float32)
        bins = np.stack([rng.integers(-2, 23, Bz), rng.integers(-1, 6, Bz)], 1).astype(np.int32)
        budget = 300
        cap = min(T, budget * Hkv - (Hkv - 1) * W)
        p = B.make_params(batch=Bz, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128, seq_len=T, window=W,
                          dtype="bf16", pool=pool, pool_kernel=kernel, budget=budget, cap=cap, layer=2,
                          n_layers=n_layers, flags=B.FLAG_VALUE_NORM if vn else 0)
        dev = lambda a: torch.from_numpy(a).to(DEV)
        util = torch.full((Bz, Hkv, T - W), float("nan"), device=DEV)
        bud = torch.zeros(Bz, Hkv, dtype=torch.int32, device=DEV)
        tau = torch.zeros(Bz, device=DEV)
        B.ckv_apply_tables(p, dev(s), dev(rho) if vn else None, dev(w_head), dev(share), dev(gate), 20, 4,
                           dev(bins), util, bud, tau)
        torch.cuda.synchronize()
        ref_u = oracle.utility(s.astype(np.float64), W, Hkv, pool, kernel, w_head[2],
                               rho.astype(np.float64) if vn else None)
        np.testing.assert_allclose(util.cpu().numpy(), ref_u, rtol=1e-5, atol=0)
        ref_b = oracle.budgets(Hkv, T, W, budget, share[2])
        np.testing.assert_array_equal(bud.cpu().numpy(), np.tile(ref_b, (Bz, 1)))
        ref_tau = [oracle.tau(gate[2], bins[b, 0], bins[b, 1]) for b in range(Bz)]
        np.testing.assert_array_equal(tau.cpu().numpy(), np.array(ref_tau, np.float32))


def test_budget_rule_matches_oracle_on_skewed_shares():
    rng = np.random.default_rng(6)
    for trial in range(40):
        Hkv = int(rng.integers(1, 17))
        W = int(rng.integers(1, 65))
        Bn = W + int(rng.integers(0, 400))
        T = max(W + 1, int(rng.integers(W, 5000)))
        share = (rng.random(Hkv) ** 6).astype(np.float32) + 1e-4
        share = (share / share.sum()).astype(np.float32)[None]
        cap = min(T, Bn * Hkv - (Hkv - 1) * W)
        p = B.make_params(batch=1, n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=128, seq_len=T, window=W,
                          dtype="bf16", pool=wl.POOL_NONE, pool_kernel=1, budget=Bn, cap=cap)
        s = torch.ones(1, Hkv, T, device=DEV)
        util = torch.empty(1, Hkv, max(T - W, 1), device=DEV)
        bud = torch.zeros(1, Hkv, dtype=torch.int32, device=DEV)
        tau = torch.zeros(1, device=DEV)
        B.ckv_apply_tables(p, s, None, torch.ones(1, Hkv, device=DEV), torch.from_numpy(share).to(DEV), None,
                           0, 0, None, util, bud, tau)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bud.cpu().numpy()[0], oracle.budgets(Hkv, T, W, Bn, share[0]))


def _select_case(u, tau, budget, W, cap, with_workspace=False):
    Bz, Hkv, P = u.shape
    p = B.make_params(batch=Bz, n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=128, seq_len=P + W, window=W,
                      dtype="bf16", pool=wl.POOL_NONE, pool_kernel=1, budget=W, cap=cap)
    idx = torch.full((Bz, Hkv, cap), -1, dtype=torch.int32, device=DEV)
    cnt = torch.zeros(Bz, Hkv, dtype=torch.int32, device=DEV)
    ut = torch.from_numpy(u).to(DEV) if u.size else torch.zeros(1, device=DEV)   # P = 0: never read
    ws = None
    if with_workspace:  # filled with ones: the selection must clear what it accumulates into
        ws = torch.full((B.ckv_workspace_bytes(p),), 0x5A, dtype=torch.uint8, device=DEV)
    B.ckv_select_topk(p, ut, torch.from_numpy(budget).to(DEV),
                      torch.from_numpy(tau).to(DEV), idx, cnt, ws)
    torch.cuda.synchronize()
    oi, oc = oracle.select(u, tau, budget, W, cap)
    np.testing.assert_array_equal(cnt.cpu().numpy(), oc)
    np.testing.assert_array_equal(idx.cpu().numpy(), oi)     # entries beyond count stay -1 on both sides


def test_select_exact_including_ties_and_elastic_pool():
    rng = np.random.default_rng(7)
    # heavy ties: utilities drawn from 12 distinct values
    u = rng.choice(np.linspace(0, 2, 12).astype(np.float32), size=(2, 3, 5000))
    _select_case(u, np.array([0.0, 0.9], np.float32), rng.integers(16, 600, (2, 3)).astype(np.int32), 16, 700)
    # all equal (every radix pass sees one bin), zeros, and -0.0
    _select_case(np.full((1, 2, 3000), 0.75, np.float32), np.zeros(1, np.float32),
                 np.array([[100, 3016]], np.int32), 16, 3016)
    z = np.zeros((1, 2, 1000), np.float32)
    z[0, 1, ::3] = -0.0
    _select_case(z, np.zeros(1, np.float32), np.array([[50, 60]], np.int32), 8, 64)
    # elastic pool: thresholds that leave fewer candidates than the budget, none, or all
    u = rng.random((4, 2, 4097)).astype(np.float32)
    _select_case(u, np.array([0.999, 2.0, 0.0, 0.5], np.float32), np.full((4, 2), 300, np.int32), 32, 300)
    # kp = 0 (budget == W), budget above cap (clamped), P = 0, P < 64, distinct huge/small magnitudes
    _select_case(u, np.zeros(4, np.float32), np.array([[32, 33]] * 4, np.int32), 32, 64)
    _select_case(u, np.zeros(4, np.float32), np.full((4, 2), 100000, np.int32), 32, 500)
    _select_case(np.zeros((1, 1, 0), np.float32), np.zeros(1, np.float32), np.array([[8]], np.int32), 8, 8)
    _select_case(rng.random((2, 2, 37)).astype(np.float32), np.zeros(2, np.float32),
                 np.array([[10, 45], [7, 20]], np.int32), 4, 41)
    wide = (10.0 ** rng.uniform(-30, 30, (1, 2, 20000))).astype(np.float32)
    _select_case(wide, np.zeros(1, np.float32), np.array([[512, 1024]], np.int32), 32, 1024)
    # values that differ only in the low mantissa bits (last radix pass decides)
    base = np.float32(1.0)
    near = (base + np.arange(8000, dtype=np.float32) % 97 * np.float32(1.2e-7)).reshape(1, 1, -1)
    _select_case(near.astype(np.float32), np.zeros(1, np.float32), np.array([[333]], np.int32), 32, 400)


def test_select_long_context_unit():
    rng = np.random.default_rng(8)
    u = (rng.standard_normal((1, 2, 131072 - 64)) ** 2).astype(np.float32)
    _select_case(u, np.array([0.8], np.float32), np.array([[512, 700]], np.int32), 64, 1024)


def test_select_split_over_workgroups_long_prefixes():
    """Prefixes beyond 65536 positions with a workspace: several workgroups per unit, same unique result."""
    rng = np.random.default_rng(9)
    one, zero = np.ones(1, np.float32), np.zeros(1, np.float32)
    u = (rng.standard_normal((1, 2, 131072 - 64)) ** 2).astype(np.float32)
    _select_case(u, 0.8 * one, np.array([[512, 700]], np.int32), 64, 1024, True)
    _select_case(u, zero, np.array([[2048, 16160]], np.int32), 32, 16160, True)
    # ragged last slice, heavy ties, budgets from kp = 0 to beyond the cap
    t = rng.choice(np.linspace(0, 2, 12).astype(np.float32), size=(2, 3, 70000))
    _select_case(t, np.array([0.0, 0.9], np.float32), np.array([[16, 17, 600], [40000, 70016, 999999]], np.int32),
                 16, 70016, True)
    # all equal: every digit histogram has one bin; the position order decides
    _select_case(np.full((1, 2, 65540), 0.75, np.float32), zero, np.array([[100, 65556]], np.int32), 16, 65556, True)
    # elastic pool: fewer candidates than the budget, none, all
    v = rng.random((4, 1, 90000)).astype(np.float32)
    _select_case(v, np.array([0.9999, 2.0, 0.0, 0.5], np.float32), np.full((4, 1), 300, np.int32), 32, 300, True)
    # values that differ only in the low mantissa bits, 25 slices
    near = (np.float32(1.0) + np.arange(200000, dtype=np.float32) % 97 * np.float32(1.2e-7)).reshape(1, 1, -1)
    _select_case(near.astype(np.float32), zero, np.array([[50032]], np.int32), 32, 50032, True)
    # a prefix length that is not a multiple of four takes the streaming kernel, workspace or not
    _select_case(rng.random((1, 1, 70001)).astype(np.float32), zero, np.array([[777]], np.int32), 32, 800, True)


def test_gather_identity_and_determinism():
    w = _small("gather", "bf16", 2, 4, 2, 128, 600, 32)
    layer = wl.make_layer(w, 0, DEV)
    p = params_of(w, layer["q"], layer["k"], layer["v"], cap=600)
    p.budget_per_kv_head = 300
    idx = torch.arange(600, dtype=torch.int32, device=DEV).expand(2, 2, 600).contiguous()
    cnt = torch.full((2, 2), 600, dtype=torch.int32, device=DEV)
    ko, vo = torch.zeros_like(layer["k"]), torch.zeros_like(layer["v"])
    B.ckv_compact_kv(p, layer["k"], layer["v"], idx, cnt, ko, vo)
    torch.cuda.synchronize()
    assert torch.equal(ko, layer["k"]) and torch.equal(vo, layer["v"])
    # rows at and beyond count stay untouched; out-of-range indices are skipped
    idx[0, 0, 5] = 600
    idx[0, 0, 6] = -3
    cnt[:] = 10
    ko.fill_(7.0)
    vo.fill_(7.0)
    B.ckv_compact_kv(p, layer["k"], layer["v"], idx, cnt, ko, vo)
    torch.cuda.synchronize()
    assert torch.equal(ko[:, :, 10:], torch.full_like(ko[:, :, 10:], 7.0))
    assert torch.equal(ko[0, 0, 5:7], torch.full_like(ko[0, 0, 5:7], 7.0))
    assert torch.equal(ko[1, 1, :10], layer["k"][1, 1, :10])


def test_two_runs_are_bit_identical():
    w = wl.C2.scaled(n_q_heads=8, n_kv_heads=8)
    layer, tabs = wl.make_layer(w, 0, DEV), wl.make_tables(w, DEV)
    _, a = run_gpu(w, layer, tabs, flags=B.FLAG_VALUE_NORM)
    _, b = run_gpu(w, layer, tabs, flags=B.FLAG_VALUE_NORM)
    for name in ("scores", "vnorm_ratio", "utility", "idx", "count", "k_out", "v_out"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name


def test_outputs_stay_inside_their_buffers():
    # canaries on both sides of every output of the chain
    w = _small("canary", "bf16", 1, 8, 2, 128, 1500, 32, shares=True)
    layer, tabs = wl.make_layer(w, 0, DEV), wl.make_tables(w, DEV)
    p = params_of(w, layer["q"], layer["k"], layer["v"], flags=B.FLAG_VALUE_NORM)
    buf = B.LayerBuffers(p, DEV)
    pad = 1024
    guarded = {}
    for name in ("scores", "vnorm_ratio", "utility", "budget", "tau", "idx", "count", "k_out", "v_out"):
        t = getattr(buf, name)
        raw = torch.full((t.numel() + 2 * pad,), 1, dtype=t.dtype, device=DEV)
        guarded[name] = raw
        setattr(buf, name, raw[pad:pad + t.numel()].view(t.shape))
    B.retention_layer(p, layer["q"], layer["k"], layer["v"], tabs, buf)
    torch.cuda.synchronize()
    for name, raw in guarded.items():
        assert (raw[:pad] == 1).all() and (raw[-pad:] == 1).all(), name
