"""Pins for the oracle's observation-window scan and value-norm ratio (CPU only).

Each test checks the oracle against something other than itself: a closed form, an invariant the
paper states, a library routine on a special case, or brute force in pure Python.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def test_mass_sums_to_T():
    # Paper Eq. 4 remark: sum_t sum_{j in Omega} A[j,t] = W, so the (T/W)-scaled mass sums to T.
    q, k = _rand((2, 4, 8, 16), 1), _rand((2, 2, 100, 16), 2, 2.0)
    s = oracle.window_scores(q, k)
    assert s.shape == (2, 4, 100)
    np.testing.assert_allclose(s.sum(-1), 100.0, rtol=1e-12)
    assert (s > 0).all()


def test_constant_keys_closed_form():
    # Equal keys => every visible key of window row j gets 1/(P+j+1):
    # s[t] = (T/W) * sum_{j : P+j >= t} 1/(P+j+1). The window columns pin the causal mask.
    T, W, d = 37, 5, 8
    P = T - W
    q = _rand((1, 1, W, d), 3)
    k = np.tile(_rand((1, 1, 1, d), 4), (1, 1, T, 1))
    s = oracle.window_scores(q, k)[0, 0]
    for t in range(T):
        expect = (T / W) * sum(1.0 / (P + j + 1) for j in range(W) if P + j >= t)
        assert s[t] == pytest.approx(expect, rel=1e-12)


def test_single_row_window_is_library_softmax():
    # W = 1: the mass is T * softmax(q K^T * scale) over all T keys.
    T, d = 64, 32
    q, k = _rand((1, 1, 1, d), 5), _rand((1, 1, T, d), 6)
    s = oracle.window_scores(q, k, scale=0.37)[0, 0]
    z = torch.from_numpy(k[0, 0]).double() @ torch.from_numpy(q[0, 0, 0]).double() * 0.37
    np.testing.assert_allclose(s, T * torch.softmax(z, 0).numpy(), rtol=1e-12)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (6, 2), (8, 1)])
def test_against_library_masked_softmax(Hq, Hkv):
    # Library matmul + softmax in fp64 with an explicit causal mask; distinct K per KV head pins the
    # GQA head -> KV-head map, random Q/K pin operand order and the scale.
    Bz, W, T, d = 2, 7, 53, 16
    P, G = T - W, Hq // Hkv
    q, k = _rand((Bz, Hq, W, d), 7), _rand((Bz, Hkv, T, d), 8, 1.5)
    s, lse = oracle.window_scores(q, k, return_lse=True)
    qt = torch.from_numpy(q).double()
    kt = torch.from_numpy(k).double().repeat_interleave(G, dim=1)
    z = qt @ kt.transpose(-1, -2) / math.sqrt(d)
    mask = torch.arange(T)[None, :] > (P + torch.arange(W))[:, None]
    z = z.masked_fill(mask, -math.inf)
    ref = torch.softmax(z, -1).sum(-2) * (T / W)
    np.testing.assert_allclose(s, ref.numpy(), rtol=1e-11, atol=1e-300)
    np.testing.assert_allclose(lse, torch.logsumexp(z, -1).numpy(), rtol=1e-12)


def test_brute_force_python_loops():
    Bz, Hq, Hkv, W, T, d = 1, 2, 1, 3, 9, 4
    P = T - W
    q, k = _rand((Bz, Hq, W, d), 9), _rand((Bz, Hkv, T, d), 10)
    s = oracle.window_scores(q, k)
    for h in range(Hq):
        col = [0.0] * T
        for j in range(W):
            z = [sum(float(q[0, h, j, c]) * float(k[0, 0, t, c]) for c in range(d)) / math.sqrt(d)
                 for t in range(P + j + 1)]
            den = sum(math.exp(x) for x in z)
            for t, x in enumerate(z):
                col[t] += math.exp(x) / den
        for t in range(T):
            assert s[0, h, t] == pytest.approx(col[t] * T / W, rel=1e-12)


def test_large_logits_do_not_overflow():
    # Keys scaled 40x (logits in the hundreds): the result must stay finite and still sum to T.
    q, k = _rand((1, 2, 4, 16), 11), _rand((1, 2, 40, 16), 12, 40.0)
    s = oracle.window_scores(q, k)
    assert np.isfinite(s).all()
    np.testing.assert_allclose(s.sum(-1), 40.0, rtol=1e-12)


def test_entropy_distribution_two_definitions_agree():
    # Paper Eq. 7 defines A'_t as the (window, layer, head) mean of A; Alg. 1 as alpha / ||alpha||_1.
    # With alpha taken as the head-mean of the per-head mass both equal alpha / T.
    q, k = _rand((1, 4, 6, 8), 13), _rand((1, 2, 30, 8), 14)
    s = oracle.window_scores(q, k)[0]          # [Hq, T], each (T/W) * sum_j A
    alpha = s.mean(0)
    a_alg = alpha / np.abs(alpha).sum()
    a_eq7 = (s * (6 / 30)).sum(0) / (6 * 4)    # (1/(|Omega| H)) sum_{j,h} A
    np.testing.assert_allclose(a_alg, a_eq7, rtol=1e-12)
    assert a_alg.sum() == pytest.approx(1.0, rel=1e-12)


def test_value_norm_ratio_unit_rows_and_scale_invariance():
    v = _rand((2, 3, 50, 16), 15)
    unit = v / np.linalg.norm(v.astype(np.float64), axis=-1, keepdims=True)
    rho_unit = oracle.value_norm_ratio(unit.astype(np.float32), eps=1e-6)
    np.testing.assert_allclose(rho_unit, 1.0 / (1.0 + 1e-6), rtol=1e-6)
    # Eq. 4: the ratio removes a head's scale; with eps = 0 it is exactly invariant (power of two scale).
    a = oracle.value_norm_ratio(v, eps=0.0)
    b = oracle.value_norm_ratio(v * 8.0, eps=0.0)
    np.testing.assert_allclose(a, b, rtol=1e-13)
    np.testing.assert_allclose(a.mean(-1), 1.0, rtol=1e-12)
    # against the library norm
    r = np.linalg.norm(v.astype(np.float64), axis=-1)
    np.testing.assert_allclose(oracle.value_norm_ratio(v, eps=1e-6), r / (r.mean(-1, keepdims=True) + 1e-6),
                               rtol=1e-12)


def test_rejects_bad_shapes():
    with pytest.raises(RuntimeError):
        oracle.window_scores(_rand((1, 3, 2, 4), 1), _rand((1, 2, 8, 4), 2))   # Hq % Hkv != 0
    with pytest.raises(RuntimeError):
        oracle.window_scores(_rand((1, 2, 9, 4), 1), _rand((1, 2, 8, 4), 2))   # W > T
