"""Pins for the oracle's pooling, table application, budgets, selection and gather (CPU only)."""
import itertools
import pathlib

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

GOLDEN = pathlib.Path(__file__).parent / "golden"


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- pooling -------------------------
@pytest.mark.parametrize("kernel", [1, 3, 5, 7])
def test_pool_matches_library(kernel):
    x = _rng(1).random((3, 41))
    xt = torch.from_numpy(x)[None]
    avg = F.avg_pool1d(xt, kernel, stride=1, padding=kernel // 2, count_include_pad=True)[0]
    mx = F.max_pool1d(xt, kernel, stride=1, padding=kernel // 2)[0]
    np.testing.assert_allclose(oracle.pool(x, oracle.POOL_AVG, kernel), avg.numpy(), rtol=1e-13)
    np.testing.assert_array_equal(oracle.pool(x, oracle.POOL_MAX, kernel), mx.numpy())
    np.testing.assert_array_equal(oracle.pool(x, oracle.POOL_NONE, kernel), x)


def test_pool_hand_cases_at_edges():
    x = np.array([7.0, 0.0, 0.0, 0.0, 0.0, 0.0, 14.0])
    np.testing.assert_allclose(oracle.pool(x, oracle.POOL_AVG, 7), [1, 1, 1, 3, 2, 2, 2])
    np.testing.assert_array_equal(oracle.pool(x, oracle.POOL_MAX, 3), [7, 7, 0, 0, 0, 14, 14])
    np.testing.assert_array_equal(oracle.pool(np.array([5.0]), oracle.POOL_MAX, 7), [5.0])
    np.testing.assert_allclose(oracle.pool(np.array([5.0, 2.0]), oracle.POOL_AVG, 5), [1.4, 1.4])


# ---------------------------------------------------------------- utility -------------------------
def test_utility_identity_when_tables_neutral():
    s = _rng(2).random((2, 4, 30))
    u = oracle.utility(s, W=6, n_kv_heads=4, mode=oracle.POOL_NONE, kernel=1, w_head_row=np.ones(4))
    np.testing.assert_array_equal(u, s[:, :, :24].astype(np.float32))


def test_utility_group_max_and_veto():
    # Paper Eq. 6: a single head with a large weight decides every max of its group.
    Bz, Hq, Hkv, T, W = 1, 6, 2, 20, 4
    s = _rng(3).random((Bz, Hq, T)) + 0.1
    w = np.ones(Hq, dtype=np.float32)
    w[4] = 1000.0
    u = oracle.utility(s, W, Hkv, oracle.POOL_NONE, 1, w)
    np.testing.assert_array_equal(u[0, 1], (s[0, 4, :16] * 1000.0).astype(np.float32))
    np.testing.assert_array_equal(u[0, 0], s[0, 0:3, :16].max(0).astype(np.float32))


def test_utility_against_library_chain():
    Bz, Hq, Hkv, T, W, kernel = 2, 8, 2, 64, 8, 5
    P, G = T - W, Hq // Hkv
    s, rho = _rng(4).random((Bz, Hq, T)), _rng(5).random((Bz, Hkv, T)) + 0.5
    w = (_rng(6).random(Hq) + 0.5).astype(np.float32)
    for mode in (oracle.POOL_AVG, oracle.POOL_MAX):
        u = oracle.utility(s, W, Hkv, mode, kernel, w, rho)
        st = torch.from_numpy(s[:, :, :P])
        pooled = (F.avg_pool1d(st, kernel, 1, kernel // 2, count_include_pad=True) if mode == oracle.POOL_AVG
                  else F.max_pool1d(st, kernel, 1, kernel // 2))
        full = pooled * torch.from_numpy(rho[:, :, :P]).repeat_interleave(G, 1) * torch.from_numpy(w).double()[None, :, None]
        ref = full.view(Bz, Hkv, G, P).max(2).values.float().numpy()
        np.testing.assert_allclose(u, ref, rtol=2e-7)


# ---------------------------------------------------------------- budgets / gate ------------------
def test_budgets_hand_example():
    # B_tot = 256: floor -> [179,25,25,25]; floor W=32 -> [179,32,32,32] (275); the largest loses 19.
    share = np.array([0.7, 0.1, 0.1, 0.1], dtype=np.float32)
    np.testing.assert_array_equal(oracle.budgets(4, 1024, 32, 64, share), [160, 32, 32, 32])
    # ties: lowest head loses first; two leaders level off together
    share = np.array([0.45, 0.45, 0.05, 0.05], dtype=np.float32)
    out = oracle.budgets(4, 1024, 32, 64, share)      # [115,115,32,32] = 294 -> lose 38 -> 96,96
    np.testing.assert_array_equal(out, [96, 96, 32, 32])
    share = np.array([0.5, 0.49, 0.005, 0.005], dtype=np.float32)   # [128,125,32,32]=317 -> lose 61
    np.testing.assert_array_equal(oracle.budgets(4, 1024, 32, 64, share), [96, 96, 32, 32])
    # clamp to T
    np.testing.assert_array_equal(oracle.budgets(2, 40, 8, 30, np.array([0.9, 0.1], dtype=np.float32)), [40, 8])


def test_budgets_invariants_random():
    r = _rng(7)
    for _ in range(200):
        Hkv = int(r.integers(1, 9))
        W = int(r.integers(1, 40))
        B = W + int(r.integers(0, 200))
        T = W + int(r.integers(0, 2000))
        share = r.random(Hkv).astype(np.float32)
        share /= share.sum()
        b = oracle.budgets(Hkv, T, W, B, share)
        assert (b >= W).all() and (b <= T).all() and b.sum() <= B * Hkv
        want = np.clip(np.floor(share.astype(np.float64) * (B * Hkv)), W, T).astype(np.int64)
        if want.sum() <= B * Hkv:
            np.testing.assert_array_equal(b, want)      # no correction needed
        else:
            cut = want - b
            assert (cut >= 0).all() and b.sum() == B * Hkv
            level = b[cut > 0].max()                    # heads that lost tokens end within 1 of a common level
            assert (b[cut > 0] >= level - 1).all() or (b[cut > 0] == W).any()
            assert (b[cut == 0] <= level).all()
    np.testing.assert_array_equal(oracle.budgets(5, 4096, 32, 512, None), [512] * 5)
    uniform = np.full(4, 0.25, dtype=np.float32)
    np.testing.assert_array_equal(oracle.budgets(4, 4096, 32, 512, uniform), [512] * 4)


def test_gate_lookup_and_table_shape():
    # Paper App. "Offline Table Compilation": 32 x 20 x 4 = 2560 entries, 21 tau levels in [0.8, 1.0].
    lines = dict(l.split("=") for l in (GOLDEN / "table_shapes.txt").read_text().split() if "=" in l)
    assert int(lines["layers"]) * int(lines["entropy_bins"]) * int(lines["ppl_bins"]) == int(lines["lut_entries"]) == 2560
    levels = np.linspace(float(lines["tau_min"]), float(lines["tau_max"]), int(lines["tau_levels"]))
    assert levels[1] - levels[0] == pytest.approx(0.01)
    gate = np.arange(80, dtype=np.float32).reshape(20, 4)
    assert oracle.tau(gate, 3, 2) == 14.0
    assert oracle.tau(gate, 99, -1) == 76.0     # clamped into the table
    assert oracle.tau(None, 0, 0) == 0.0


# ---------------------------------------------------------------- selection -----------------------
def _brute_force_select(u, tau, kp):
    """Max-total-utility subset of the candidates, size min(kp, #cand); unique for distinct utilities."""
    cand = [t for t in range(len(u)) if u[t] >= tau]
    if len(cand) <= kp:
        return cand
    best = max(itertools.combinations(cand, kp), key=lambda c: sum(float(u[t]) for t in c))
    return sorted(best)


def test_select_brute_force_tiny():
    r = _rng(8)
    for trial in range(60):
        P, W = int(r.integers(1, 11)), int(r.integers(1, 4))
        T = P + W
        u = r.permutation(P).astype(np.float32)[None, None] * 0.25 + 0.125      # distinct values
        tau = np.array([r.choice([0.0, 0.6, 1.3, 99.0])], dtype=np.float32)
        budget = np.array([[W + int(r.integers(0, P + 1))]], dtype=np.int32)
        idx, count = oracle.select(u, tau, budget, W, cap=T)
        keep = _brute_force_select(u[0, 0], float(tau[0]), int(budget[0, 0]) - W)
        assert count[0, 0] == len(keep) + W
        assert idx[0, 0, : count[0, 0]].tolist() == keep + list(range(P, T))
        assert (idx[0, 0, count[0, 0]:] == -1).all()


def test_select_matches_library_topk_when_gate_off():
    Bz, Hkv, P, W, B = 2, 3, 500, 16, 80
    u = _rng(9).random((Bz, Hkv, P)).astype(np.float32)
    idx, count = oracle.select(u, np.zeros(Bz, np.float32), np.full((Bz, Hkv), B, np.int32), W, cap=B)
    top = torch.topk(torch.from_numpy(u), B - W, dim=-1).indices.sort(-1).values.numpy()
    assert (count == B).all()
    np.testing.assert_array_equal(idx[:, :, : B - W], top)
    np.testing.assert_array_equal(idx[:, :, B - W:], np.broadcast_to(np.arange(P, P + W), (Bz, Hkv, W)))


def test_select_ties_take_lowest_positions():
    u = np.array([[[1.0, 2.0, 1.0, 1.0, 2.0, 1.0, 0.5]]], dtype=np.float32)
    idx, count = oracle.select(u, np.zeros(1, np.float32), np.array([[2 + 4]], np.int32), 2, cap=9)
    assert count[0, 0] == 6 and idx[0, 0, :6].tolist() == [0, 1, 2, 4, 7, 8]


def test_select_elastic_pool_and_window_only():
    # Paper Eq. 8: fewer candidates than the budget => keep exactly the candidates (inclusive >=).
    u = np.array([[[0.9, 0.2, 0.8, 0.79999, 1.5]]], dtype=np.float32)
    tau = np.array([0.8], dtype=np.float32)
    idx, count = oracle.select(u, tau, np.array([[3 + 4]], np.int32), 3, cap=8)
    assert count[0, 0] == 3 + 3 and idx[0, 0, :6].tolist() == [0, 2, 4, 5, 6, 7]
    idx, count = oracle.select(u, np.array([2.0], np.float32), np.array([[7]], np.int32), 3, cap=8)
    assert count[0, 0] == 3 and idx[0, 0, :3].tolist() == [5, 6, 7]
    # count = min(budget, W + #cand) on random inputs; window always last
    r = _rng(10)
    u = r.random((4, 2, 300)).astype(np.float32)
    tau = np.array([0.0, 0.5, 0.9, 0.99], dtype=np.float32)
    bud = r.integers(8, 120, (4, 2)).astype(np.int32)
    idx, count = oracle.select(u, tau, bud, 8, cap=128)
    ncand = (u >= tau[:, None, None]).sum(-1)
    np.testing.assert_array_equal(count, np.minimum(bud, 8 + ncand))
    for b in range(4):
        for g in range(2):
            c = count[b, g]
            assert idx[b, g, c - 8:c].tolist() == list(range(300, 308))
            assert (np.diff(idx[b, g, :c]) > 0).all()


def test_retention_ratios_of_the_paper():
    # Paper Table A6: budget 512 keeps 6.25 % / 3.12 % / 1.56 % of an 8k / 16k / 32k prefill.
    for line in (GOLDEN / "retention_ratios.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        T, B, pct = line.split()
        T, B = int(T), int(B)
        u = _rng(T).random((1, 1, T - 32)).astype(np.float32)
        _, count = oracle.select(u, np.zeros(1, np.float32), np.array([[B]], np.int32), 32, cap=B)
        # the paper prints two decimals, truncated (3.125 -> 3.12, 1.5625 -> 1.56)
        assert int(100 * 100.0 * count[0, 0] / T) / 100 == float(pct)


# ---------------------------------------------------------------- gather --------------------------
def test_gather_matches_library_and_identity():
    r = _rng(11)
    src = r.integers(-2**15, 2**15, (2, 3, 40, 8)).astype(np.int16)      # raw bf16 bit patterns
    idx = np.sort(r.integers(0, 40, (2, 3, 12)), axis=-1).astype(np.int32)
    count = r.integers(0, 13, (2, 3)).astype(np.int32)
    out = oracle.gather(src, idx, count)
    ref = np.take_along_axis(src, idx[..., None].astype(np.int64), axis=2)
    for b in range(2):
        for g in range(3):
            c = count[b, g]
            np.testing.assert_array_equal(out[b, g, :c], ref[b, g, :c])
            assert (out[b, g, c:] == 0).all()
    ident = np.broadcast_to(np.arange(40, dtype=np.int32), (2, 3, 40)).copy()
    np.testing.assert_array_equal(oracle.gather(src, ident, np.full((2, 3), 40, np.int32)), src)
    with pytest.raises(RuntimeError):
        oracle.gather(src, np.full((2, 3, 1), 40, np.int32), np.ones((2, 3), np.int32))
