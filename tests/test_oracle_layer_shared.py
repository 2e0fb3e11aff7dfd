"""Pins of the oracle's layer-shared mode (Alg. 1 as printed): what the paper and the mathematics fix,
against closed forms, library routines and brute force."""
import numpy as np
import scipy.stats

import oracle


def test_alpha_is_the_mean_over_layers_and_heads_and_keeps_mean_one():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((2, 4, 8, 16)).astype(np.float32)
    maps = []
    for layer in range(3):
        k = rng.standard_normal((2, 2, 50, 16)).astype(np.float32)
        maps.append(oracle.window_scores(q, k))
    a = oracle.alpha_mean(maps)
    assert a.shape == (2, 50)
    np.testing.assert_allclose(a.sum(-1), 50.0, rtol=1e-12)                   # Eq. 4: mean scale one
    brute = sum(m[:, h] for m in maps for h in range(4)) / 12.0
    np.testing.assert_allclose(a, brute, rtol=1e-13)
    np.testing.assert_allclose(oracle.alpha_mean(maps[:1])[:, :] * 4, maps[0].sum(1), rtol=1e-13)   # L = 1


def test_risk_struct_closed_forms_and_library():
    T = 64
    np.testing.assert_allclose(oracle.risk_struct(np.full((1, T), 3.7)), np.log(T), rtol=1e-13)      # uniform
    one = np.zeros((1, T))
    one[0, 5] = 9.0
    assert oracle.risk_struct(one)[0] == 0.0                                                          # a single focal point
    p = 0.3
    two = np.zeros((1, T))
    two[0, 1], two[0, 9] = p, 1 - p
    np.testing.assert_allclose(oracle.risk_struct(two), -p * np.log(p) - (1 - p) * np.log(1 - p), rtol=1e-13)
    rng = np.random.default_rng(1)
    a = rng.random((3, 200)) ** 3
    np.testing.assert_allclose(oracle.risk_struct(a), scipy.stats.entropy(a, axis=-1), rtol=1e-12)    # library routine
    np.testing.assert_allclose(oracle.risk_struct(5.0 * a), oracle.risk_struct(a), rtol=1e-12)        # scale-free
    # Eq. 7's A' (mean of A over the window, layers and heads) is alpha / T, and alpha sums to T
    a = a / a.sum(-1, keepdims=True) * 200
    np.testing.assert_allclose(oracle.risk_struct(a), scipy.stats.entropy(a / 200, axis=-1), rtol=1e-12)


def test_discretize():
    edges = [0.5, 1.0, 2.0]
    assert oracle.discretize([0.1, 0.5, 0.99, 1.0, 1.5, 2.0, 7.0], edges).tolist() == [0, 1, 1, 2, 2, 3, 3]
    v = np.random.default_rng(2).random(50) * 3
    np.testing.assert_array_equal(oracle.discretize(v, edges), np.searchsorted(edges, v, side="right"))
    assert oracle.discretize(1.0, []).tolist() == [0]


def test_shared_utility_special_cases_and_brute_force():
    rng = np.random.default_rng(3)
    Bz, Hq, Hkv, T, W = 2, 6, 3, 40, 8
    alpha = rng.random((Bz, T)) * 2
    rho = rng.random((Bz, Hkv, T)) + 0.5
    w = (rng.random(Hq) + 0.5).astype(np.float32)
    u = oracle.shared_utility(alpha, rho, w, W)
    assert u.shape == (Bz, T - W) and u.dtype == np.float32
    # brute force, head by head (query head h reads the value norms of KV head h // G)
    for b in range(Bz):
        for t in range(T - W):
            ref = max(np.float32(np.float64(w[h]) * alpha[b, t] * rho[b, h // 2, t]) for h in range(Hq))
            assert u[b, t] == ref
    # positive weights factor out: alpha * max_g(rho_g * max_{h in g} w_h)
    wmax = w.reshape(Hkv, 2).max(1).astype(np.float64)
    np.testing.assert_allclose(u, alpha[:, :T - W] * (rho[:, :, :T - W] * wmax[None, :, None]).max(1), rtol=1e-6)
    # one head, unit norms, unit weight: the utility is alpha itself (Eq. 4 with rho = 1)
    one = oracle.shared_utility(alpha, np.ones((Bz, 1, T)), np.ones(1, np.float32), W)
    np.testing.assert_array_equal(one, alpha[:, :T - W].astype(np.float32))
    # veto (Eq. 6): raising one head's weight far above the others makes that head's KV norms decide
    big = w.copy()
    big[4] = 100.0
    np.testing.assert_allclose(oracle.shared_utility(alpha, rho, big, W),
                               100.0 * alpha[:, :T - W] * rho[:, 2, :T - W], rtol=1e-6)


def test_gather_shared_and_whole_layer():
    rng = np.random.default_rng(4)
    Bz, Hq, Hkv, T, W, d = 2, 4, 2, 60, 6, 8
    k = rng.standard_normal((Bz, Hkv, T, d)).astype(np.float32)
    v = rng.standard_normal((Bz, Hkv, T, d)).astype(np.float32)
    idx = np.stack([np.sort(rng.choice(T, 10, replace=False)) for _ in range(Bz)]).astype(np.int32)
    cnt = np.array([10, 7], np.int32)
    out = oracle.gather_shared(k, idx, cnt)
    for b in range(Bz):
        for g in range(Hkv):
            np.testing.assert_array_equal(out[b, g, :cnt[b]], k[b, g, idx[b, :cnt[b]]])     # take along the token axis
            assert (out[b, g, cnt[b]:] == 0).all()
    alpha = rng.random((Bz, T)) + 0.2
    w = np.ones(Hq, np.float32)
    r = oracle.layer_shared_layer(alpha, k, v, v, W=W, B_layer=20, cap=20, w_head_row=w)
    assert (r["count"] == 20).all()                                     # gate off: every token is a candidate
    for b in range(Bz):
        kept = r["idx"][b, :20]
        assert kept[-W:].tolist() == list(range(T - W, T))              # the window is kept, last
        top = np.sort(np.argsort(-r["utility"][b], kind="stable")[:20 - W])
        np.testing.assert_array_equal(kept[:20 - W], top)               # plain top-k of u_hat (library sort)
    # a gate above every utility keeps the window only (elastic under-retention, Eq. 8)
    gate = np.full((3, 2), 1e9, np.float32)
    r = oracle.layer_shared_layer(alpha, k, v, v, W=W, B_layer=20, cap=20, w_head_row=w, gate_layer=gate,
                                  risk_bins=[(0, 0), (2, 1)])
    assert (r["count"] == W).all()


def test_depth_mapping_is_relative_depth_interpolation():
    rng = np.random.default_rng(5)
    t = rng.random((32, 6))
    np.testing.assert_allclose(oracle.map_table_depth(t, 32), t, rtol=1e-15)                   # same depth: identity
    for L in (28, 40, 80, 2):
        m = oracle.map_table_depth(t, L)
        np.testing.assert_allclose(m[0], t[0], rtol=1e-15)                                     # first and last layer
        np.testing.assert_allclose(m[-1], t[-1], rtol=1e-12)
        x = np.arange(L) * 31 / (L - 1)
        for c in range(6):                                                                     # library interpolation
            np.testing.assert_allclose(m[:, c], np.interp(x, np.arange(32), t[:, c]), rtol=1e-12, atol=1e-15)
    ramp = np.arange(32, dtype=np.float64)[:, None] * np.array([[1.0, -2.0]]) + 3.0
    np.testing.assert_allclose(oracle.map_table_depth(ramp, 28)[:, 0], 3.0 + np.arange(28) * 31 / 27, rtol=1e-13)  # linear tables map exactly
    mono = np.sort(rng.random((32, 3)), axis=0)
    assert (np.diff(oracle.map_table_depth(mono, 48), axis=0) >= -1e-15).all()                 # monotone in depth
    assert oracle.map_table_depth(t, 1).shape == (1, 6)
    np.testing.assert_array_equal(oracle.map_table_depth(t, 1)[0], t[0])
    g = rng.random((32, 20, 4))                                                                # gate table: trailing axes ride along
    np.testing.assert_allclose(oracle.map_table_depth(g, 28)[5], 
                               (1 - (5 * 31 / 27 - 5)) * g[5] + (5 * 31 / 27 - 5) * g[6], rtol=1e-12)
