"""Pins of the oracle's decode-side consumer: the identities and the bound of Proposition 1 (App. A),
library attention as the special case "everything retained", closed forms and brute force."""
import numpy as np
import torch

import oracle


def _case(seed, Bz=2, Hq=4, Hkv=2, Nq=5, T=70, d=16, keep=20):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((Bz, Hq, Nq, d)).astype(np.float32)
    k = (1.5 * rng.standard_normal((Bz, Hkv, T, d))).astype(np.float32)
    v = rng.standard_normal((Bz, Hkv, T, d)).astype(np.float32)
    idx = np.full((Bz, Hkv, keep + 3), -1, np.int32)
    count = np.zeros((Bz, Hkv), np.int32)
    for b in range(Bz):
        for g in range(Hkv):
            n = keep - (b + g) % 3
            idx[b, g, :n] = np.sort(rng.choice(T, n, replace=False))
            count[b, g] = n
    return q, k, v, idx, count


def test_row_l1_error_is_twice_the_discarded_mass_and_the_frobenius_bound_holds():
    q, k, v, idx, count = _case(0)
    p, pt = oracle.attention_rows(q, k, idx, count)
    m = oracle.discarded_mass(q, k, idx, count)
    assert (m > 0).all() and (m < 1).all()
    np.testing.assert_allclose(np.abs(p - pt).sum(-1), 2.0 * m, rtol=1e-12)         # proof of Prop. 1: ||p - p~||_1 = 2 m
    np.testing.assert_allclose(pt.sum(-1), 1.0, rtol=1e-12)
    Nq = q.shape[2]
    fro = np.sqrt(((p - pt) ** 2).sum((-1, -2)))                                     # per head, over the Nq rows
    eps = oracle.tail_eps(m)
    assert (fro <= 2.0 * np.sqrt(Nq) * eps * (1 + 1e-12)).all()                      # single-head bound
    assert (fro.mean(1) <= 2.0 * np.sqrt(Nq) * eps.mean(1) * (1 + 1e-12)).all()      # the Proposition's bound: head average
    np.testing.assert_allclose(eps, np.sqrt((m ** 2).sum(-1) / Nq), rtol=1e-13)


def test_everything_retained_is_library_attention_and_loses_nothing():
    q, k, v, _, _ = _case(1)
    Bz, Hkv, T, d = k.shape
    out, lse = oracle.decode_attention(q, k, v)
    G = q.shape[1] // Hkv
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double().repeat_interleave(G, 1),
        torch.from_numpy(v).double().repeat_interleave(G, 1))
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-10, atol=1e-12)
    z = torch.einsum("bhqd,bhrd->bhqr", torch.from_numpy(q).double(),
                     torch.from_numpy(k).double().repeat_interleave(G, 1)) / np.sqrt(d)
    np.testing.assert_allclose(lse, torch.logsumexp(z, -1).numpy(), rtol=1e-12)
    full_idx = np.tile(np.arange(T, dtype=np.int32), (Bz, Hkv, 1))
    full_cnt = np.full((Bz, Hkv), T, np.int32)
    np.testing.assert_allclose(oracle.discarded_mass(q, k, full_idx, full_cnt), 0.0, atol=1e-15)


def test_compact_cache_attention_equals_the_renormalised_restriction():
    q, k, v, idx, count = _case(2)
    Bz, Hkv, T, d = k.shape
    cap = idx.shape[-1]
    kc, vc = oracle.gather(k, idx, count), oracle.gather(v, idx, count)
    out_c, lse_c = oracle.decode_attention(q, kc, vc, count)
    p, pt = oracle.attention_rows(q, k, idx, count)
    G = q.shape[1] // Hkv
    brute = np.einsum("bhqt,bhtd->bhqd", pt, np.repeat(v.astype(np.float64), G, axis=1))
    np.testing.assert_allclose(out_c, brute, rtol=1e-10, atol=1e-12)                  # p~ applied to V
    _, lse_f = oracle.decode_attention(q, k, v)
    m = oracle.discarded_mass(q, k, idx, count)
    np.testing.assert_allclose(1.0 - np.exp(lse_c - lse_f), m, rtol=1e-10)           # retained mass = exp(lse_S - lse)
    # rows of the compact cache beyond count are never read
    kc2, vc2 = kc.copy(), vc.copy()
    for b in range(Bz):
        for g in range(Hkv):
            kc2[b, g, count[b, g]:] = 1e30
            vc2[b, g, count[b, g]:] = np.nan
    out2, lse2 = oracle.decode_attention(q, kc2, vc2, count)
    np.testing.assert_array_equal(out2, out_c)
    np.testing.assert_array_equal(lse2, lse_c)


def test_closed_forms():
    # equal keys: uniform attention; dropping n of T keys discards n / T of the mass, whatever the query
    T, d = 40, 8
    q = np.random.default_rng(3).standard_normal((1, 1, 3, d)).astype(np.float32)
    k = np.tile(np.float32(0.3) * np.ones((1, 1, 1, d), np.float32), (1, 1, T, 1))
    v = np.arange(T * d, dtype=np.float32).reshape(1, 1, T, d)
    idx = np.arange(0, 30, dtype=np.int32).reshape(1, 1, 30)
    cnt = np.array([[30]], np.int32)
    np.testing.assert_allclose(oracle.discarded_mass(q, k, idx, cnt), 10 / T, rtol=1e-12)
    out, lse = oracle.decode_attention(q, k[:, :, :30], v[:, :, :30])
    np.testing.assert_allclose(out, np.broadcast_to(v[0, 0, :30].mean(0), out.shape), rtol=1e-12)
    z = (q.astype(np.float64) * np.float64(np.float32(0.3))).sum(-1) / np.sqrt(d)
    np.testing.assert_allclose(lse, z + np.log(30), rtol=1e-12)
    np.testing.assert_allclose(oracle.tail_eps(np.full((1, 1, 3), 0.25)), 0.25, rtol=1e-15)
    # one dominant key: discarding it loses (almost) everything, keeping only it loses (almost) nothing
    k2 = np.zeros((1, 1, T, d), np.float32)
    k2[0, 0, 7] = 50.0 * q[0, 0, 0] / np.linalg.norm(q[0, 0, 0])
    only = np.array([[[7]]], np.int32)
    rest = np.array([[[t for t in range(T) if t != 7]]], np.int32)
    m_only = oracle.discarded_mass(q[:, :, :1], k2, only, np.array([[1]], np.int32))
    m_rest = oracle.discarded_mass(q[:, :, :1], k2, rest, np.array([[T - 1]], np.int32))
    assert m_only[0, 0, 0] < 1e-6 and m_rest[0, 0, 0] > 1 - 1e-6
    np.testing.assert_allclose(m_only + m_rest, 1.0, rtol=1e-12)
