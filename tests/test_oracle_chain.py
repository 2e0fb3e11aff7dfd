"""Whole-chain pins for the oracle on the small workload (CPU only): the invariants the method and
its workload definition fix, an independent library implementation of the neutral-table case, and
the paper's exact row identity for attention over a compacted cache."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2602_08686_amd import workloads as wl


def _f32(t):
    return t.to(torch.float32).numpy()


@pytest.fixture(scope="module")
def c1():
    w = wl.C1
    layer, tabs = wl.make_layer(w, 0), wl.make_tables(w)
    out = oracle.retention_layer(
        _f32(layer["q"]), _f32(layer["k"]), _f32(layer["v"]), W=w.window, mode=w.pool,
        kernel=w.pool_kernel, B=w.budget, cap=w.cap, w_head_row=tabs["w_head"][0].numpy(),
        share_row=tabs["head_share"][0].numpy())
    return w, layer, tabs, out


def test_window_always_kept_and_count_is_clamped_budget(c1):
    w, _, _, out = c1
    P, T, W = w.prefix, w.seq_len, w.window
    assert out["budget"].sum() <= w.budget * w.n_kv_heads
    for g in range(w.n_kv_heads):
        c = out["count"][0, g]
        assert c == out["budget"][0, g]          # gate off => every prefix token is a candidate
        assert out["idx"][0, g, c - W:c].tolist() == list(range(P, T))
        assert (np.diff(out["idx"][0, g, :c]) > 0).all()


def test_planted_needles_are_retained(c1):
    w, layer, _, out = c1
    for g in range(w.n_kv_heads):
        kept = set(out["idx"][0, g, : out["count"][0, g]].tolist())
        for pos in layer["needle_pos"][0, g].tolist():
            assert pos in kept


def test_gathered_rows_are_the_selected_rows(c1):
    w, layer, _, out = c1
    k = _f32(layer["k"])
    for g in range(w.n_kv_heads):
        c = out["count"][0, g]
        np.testing.assert_array_equal(out["k_out"][0, g, :c], k[0, g, out["idx"][0, g, :c]])


def test_neutral_tables_reduce_to_observation_window_selection():
    # Weights 1, uniform budgets, gate off, no value norm: softmax -> window sum -> pool -> top-(B-W)
    # plus the window, written here with library routines only.
    w = wl.C1
    layer = wl.make_layer(w, 0)
    q, k = _f32(layer["q"]), _f32(layer["k"])
    out = oracle.retention_layer(q, k, None, W=w.window, mode=w.pool, kernel=w.pool_kernel, B=w.budget,
                                 cap=w.budget, w_head_row=np.ones(w.n_q_heads, np.float32))
    T, W, P = w.seq_len, w.window, w.prefix
    z = torch.from_numpy(q).double() @ torch.from_numpy(k).double().transpose(-1, -2) / math.sqrt(w.head_dim)
    z = z.masked_fill(torch.arange(T)[None, :] > (P + torch.arange(W))[:, None], -math.inf)
    mass = torch.softmax(z, -1).sum(-2)[..., :P]
    pooled = F.avg_pool1d(mass, w.pool_kernel, 1, w.pool_kernel // 2, count_include_pad=True)
    top = torch.topk(pooled, w.budget - W, dim=-1).indices.sort(-1).values
    np.testing.assert_array_equal(out["idx"][:, :, : w.budget - W], top.numpy())
    assert (out["count"] == w.budget).all()


def test_row_l1_identity_over_compacted_cache(c1):
    # Paper Eq. A2: for a query row p over the full cache and its renormalised restriction p~ to the
    # retained set, ||p - p~||_1 = 2 m with m the discarded mass. p~ is computed from the gathered
    # K rows, so a wrong index or a wrong gathered row breaks the identity.
    w, layer, _, out = c1
    k = torch.from_numpy(_f32(layer["k"])).double()
    qn = torch.randn(w.head_dim, generator=torch.Generator().manual_seed(7)).double()
    for g in range(w.n_kv_heads):
        c = int(out["count"][0, g])
        idx = torch.from_numpy(out["idx"][0, g, :c]).long()
        p = torch.softmax(k[0, g] @ qn / math.sqrt(w.head_dim), 0)
        pt_kept = torch.softmax(torch.from_numpy(out["k_out"][0, g, :c]).double() @ qn / math.sqrt(w.head_dim), 0)
        pt = torch.zeros_like(p)
        pt[idx] = pt_kept
        m = 1.0 - p[idx].sum()
        assert float((p - pt).abs().sum()) == pytest.approx(2.0 * float(m), rel=1e-9)


def test_gate_shrinks_pool_and_value_norm_changes_only_through_rho():
    w = wl.C1.scaled(seq_len=256, budget=64)
    layer = wl.make_layer(w, 0)
    q, k, v = _f32(layer["q"]), _f32(layer["k"]), _f32(layer["v"])
    gate = np.full((20, 4), 0.8, np.float32)
    gate[5, 1] = 1.0e9
    ones = np.ones(w.n_q_heads, np.float32)
    kw = dict(W=w.window, mode=w.pool, kernel=w.pool_kernel, B=w.budget, cap=w.cap, w_head_row=ones)
    hi = oracle.retention_layer(q, k, None, gate_layer=gate, risk_bins=[(5, 1)], **kw)
    assert (hi["count"] == w.window).all()                       # nothing passes: window only
    lo = oracle.retention_layer(q, k, None, gate_layer=gate, risk_bins=[(0, 0)], **kw)
    ncand = (lo["utility"] >= 0.8).sum(-1)
    np.testing.assert_array_equal(lo["count"], np.minimum(w.budget, w.window + ncand))
    # unit-norm values => rho = 1/(1+eps): utilities scale by that constant, selection is unchanged
    vu = (v / np.linalg.norm(v, axis=-1, keepdims=True)).astype(np.float32)
    a = oracle.retention_layer(q, k, None, **kw)
    b = oracle.retention_layer(q, k, None, v=vu, value_norm=True, **kw)
    np.testing.assert_allclose(b["utility"], a["utility"], rtol=1e-5)
    np.testing.assert_array_equal(a["idx"], b["idx"])
