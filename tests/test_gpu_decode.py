"""GPU parity of the decode-side consumer (Proposition 1): attention of decoding queries over the ragged
compact cache and over the full cache, the discarded mass and the tail epsilon, through the C ABI against
the oracle on the same tensors.

Tolerances (fp32 arithmetic on both inputs' exact values; logits are sums of d <= 128 products, the
softmax runs in the log2 domain with v_exp_f32): outputs within 1e-3 of the row's largest component
(relative 1e-3 beyond that), normalisers within 1e-4 absolute, masses within 5e-5 + 1e-3 relative."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import bits, f32, run_gpu

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _w(name, dtype, Bz, Hq, Hkv, d, T, W, budget):
    return wl.Workload(name, dtype, Bz, Hq, Hkv, d, T, W, wl.POOL_AVG, 5, budget, 2, seed=300 + T + Hq, pareto_frac=0.05)


CASES = [
    (_w("dec_bf16_gqa4", "bf16", 2, 8, 2, 128, 3001, 32, 200), 1),
    (_w("dec_bf16_mha", "bf16", 1, 4, 4, 128, 1500, 32, 100), 3),
    (_w("dec_bf16_gqa7", "bf16", 1, 7, 1, 128, 2500, 32, 300), 2),         # eight rows per sweep, one padded
    (_w("dec_bf16_gqa3_d64", "bf16", 2, 6, 2, 64, 1111, 16, 77), 1),       # three heads pad to four; 128-byte rows
    (_w("dec_bf16_gqa16", "bf16", 1, 16, 1, 128, 900, 32, 64), 1),         # two sweeps of eight heads
    (_w("dec_bf16_gqa2", "bf16", 1, 4, 2, 128, 70000, 64, 6000), 2),       # many chunks, also over the compact cache
    (_w("dec_f32_mha", "f32", 1, 4, 4, 64, 1024, 32, 128), 2),
    (_w("dec_f32_gqa2_d128", "f32", 2, 4, 2, 128, 777, 20, 60), 1),
]


def _close_rows(got, ref, what):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    tol = 1e-3 * np.maximum(np.abs(ref), np.abs(ref).max(-1, keepdims=True))
    bad = np.abs(got - ref) > tol
    assert not bad.any(), f"{what}: {bad.sum()} elements off, worst {np.abs(got - ref).max():.3e}"


def _decode(p, q_dec, k_rows, v_rows, count):
    Bz, Hq, n_q, d = q_dec.shape
    out = torch.full((Bz, Hq, n_q, d), float("nan"), device=DEV)
    lse = torch.full((Bz, Hq, n_q), float("nan"), device=DEV)
    ws = torch.empty(max(B.ckv_decode_workspace_bytes(p, n_q, k_rows.shape[2]), 256), dtype=torch.uint8, device=DEV)
    B.ckv_decode_attention(p, q_dec, k_rows, v_rows, count, out, lse, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


@pytest.mark.parametrize("w,n_q", CASES, ids=lambda x: x.name if isinstance(x, wl.Workload) else f"nq{x}")
def test_decode_over_compact_and_full_cache(w, n_q):
    print(f"case {w.name} n_q={n_q}", flush=True)
    t, tabs = wl.make_layer(w, 0, DEV), wl.make_tables(w, DEV)
    p, buf = run_gpu(w, t, tabs)
    q_dec = wl.make_decode_queries(w, 0, n_q, DEV)
    idx, count = buf.idx.cpu().numpy(), buf.count.cpu().numpy()
    # rows of the compact cache beyond count must never be read
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            buf.k_out[b, g, count[b, g]:] = 3.0e38
            buf.v_out[b, g, count[b, g]:] = float("nan")
    out_c, lse_c = _decode(p, q_dec, buf.k_out, buf.v_out, buf.count)
    ref_out_c, ref_lse_c = oracle.decode_attention(f32(q_dec), f32(buf.k_out), f32(buf.v_out), count)
    _close_rows(out_c, ref_out_c, "attention over the compact cache")
    np.testing.assert_allclose(lse_c, ref_lse_c, atol=1e-4, rtol=0)
    out_f, lse_f = _decode(p, q_dec, t["k"], t["v"], None)
    ref_out_f, ref_lse_f = oracle.decode_attention(f32(q_dec), f32(t["k"]), f32(t["v"]))
    _close_rows(out_f, ref_out_f, "attention over the full cache")
    np.testing.assert_allclose(lse_f, ref_lse_f, atol=1e-4, rtol=0)
    mass = torch.full((w.batch, w.n_q_heads, n_q), float("nan"), device=DEV)
    eps = torch.full((w.batch, w.n_q_heads), float("nan"), device=DEV)
    B.ckv_discarded_mass(p, n_q, torch.from_numpy(lse_f).to(DEV), torch.from_numpy(lse_c).to(DEV), mass, eps)
    torch.cuda.synchronize()
    ref_m = oracle.discarded_mass(f32(q_dec), f32(t["k"]), idx, count)
    np.testing.assert_allclose(mass.cpu().numpy(), ref_m, atol=5e-5, rtol=1e-3)
    np.testing.assert_allclose(eps.cpu().numpy(), oracle.tail_eps(ref_m), atol=5e-5, rtol=1e-3)
    # the identity of the Proposition's proof on the oracle's explicit rows, with the GPU's mass
    pr, pt = oracle.attention_rows(f32(q_dec), f32(t["k"]), idx, count)
    np.testing.assert_allclose(np.abs(pr - pt).sum(-1), 2.0 * mass.cpu().numpy(), atol=1e-4, rtol=1e-3)


def test_decode_edges_empty_sets_single_rows_strides():
    w = _w("dec_edges", "bf16", 2, 4, 2, 128, 300, 8, 40)
    t = wl.make_layer(w, 1, DEV)
    p = B.params_for(t["q"], t["k"], t["v"], pool=w.pool, pool_kernel=w.pool_kernel, budget=w.budget, cap=w.cap)
    q_dec = wl.make_decode_queries(w, 1, 2, DEV)
    # ragged counts including 0, 1 and all rows
    count = torch.tensor([[0, 1], [300, 17]], dtype=torch.int32, device=DEV)
    out, lse = _decode(p, q_dec, t["k"], t["v"], count)
    assert (out[0, :2] == 0).all() and np.isneginf(lse[0, :2]).all()               # KV head 0 of batch 0 is empty
    cn = count.cpu().numpy()
    for b, g in ((0, 1), (1, 0), (1, 1)):
        n = int(cn[b, g])
        ro, rl = oracle.decode_attention(f32(q_dec[b:b + 1, 2 * g:2 * g + 2]), f32(t["k"][b:b + 1, g:g + 1, :n]),
                                         f32(t["v"][b:b + 1, g:g + 1, :n]))
        _close_rows(out[b:b + 1, 2 * g:2 * g + 2], ro, f"unit ({b},{g})")
        np.testing.assert_allclose(lse[b:b + 1, 2 * g:2 * g + 2], rl, atol=1e-4, rtol=0)
    one = oracle.decode_attention(f32(q_dec[:1, 2:4]), f32(t["k"][:1, 1:2, :1]), f32(t["v"][:1, 1:2, :1]))[0]
    np.testing.assert_allclose(one, np.broadcast_to(f32(t["v"][0, 1, 0]), one.shape), rtol=1e-12)  # one row: out = v
    # K and V as slices of a fused [Bz,T,Hkv,2,d] cache; counts beyond n_rows are clamped
    kv = torch.empty(w.batch, w.seq_len, w.n_kv_heads, 2, w.head_dim, dtype=torch.bfloat16, device=DEV)
    kv[:, :, :, 0] = t["k"].transpose(1, 2)
    kv[:, :, :, 1] = t["v"].transpose(1, 2)
    ks, vs = kv[:, :, :, 0].transpose(1, 2), kv[:, :, :, 1].transpose(1, 2)
    big = torch.full((2, 2), 10 ** 6, dtype=torch.int32, device=DEV)
    out_s, lse_s = _decode(p, q_dec, ks, vs, big)
    out_f, lse_f = _decode(p, q_dec, t["k"], t["v"], None)
    np.testing.assert_array_equal(out_s, out_f)
    np.testing.assert_array_equal(lse_s, lse_f)
    # two runs are bit-identical
    out_g, lse_g = _decode(p, q_dec, t["k"], t["v"], None)
    np.testing.assert_array_equal(out_g, out_f)
    # mass: equal normalisers give zero, kept above full (rounding) clamps to zero, -inf kept gives one
    lf = torch.tensor([[[1.0, 2.0]] * 4] * 2, device=DEV)
    lk = torch.tensor([[[1.0, 2.0 + 1e-6]] * 4] * 2, device=DEV)
    lk[1, 3, 0] = float("-inf")
    mass, eps = torch.empty(2, 4, 2, device=DEV), torch.empty(2, 4, device=DEV)
    B.ckv_discarded_mass(p, 2, lf, lk, mass, eps)
    torch.cuda.synchronize()
    m = mass.cpu().numpy()
    assert m[1, 3, 0] == 1.0 and (np.delete(m.reshape(-1), 14) == 0).all()
    np.testing.assert_allclose(eps.cpu().numpy()[1, 3], np.sqrt(0.5), rtol=1e-6)


def test_decode_full_size_c3():
    """C3's shapes in the launch configuration the benchmark times: sampled units against the oracle,
    properties on everything."""
    w = wl.C3
    t, tabs = wl.make_layer(w, 0, DEV), wl.make_tables(w, DEV)
    p, buf = run_gpu(w, t, tabs)
    q_dec = wl.make_decode_queries(w, 0, 1, DEV)
    out_c, lse_c = _decode(p, q_dec, buf.k_out, buf.v_out, buf.count)
    out_f, lse_f = _decode(p, q_dec, t["k"], t["v"], None)
    mass = torch.empty(w.batch, w.n_q_heads, 1, device=DEV)
    eps = torch.empty(w.batch, w.n_q_heads, device=DEV)
    B.ckv_discarded_mass(p, 1, torch.from_numpy(lse_f).to(DEV), torch.from_numpy(lse_c).to(DEV), mass, eps)
    torch.cuda.synchronize()
    m = mass.cpu().numpy()
    assert np.isfinite(out_c).all() and np.isfinite(out_f).all()
    assert (lse_c <= lse_f + 1e-5).all() and (m >= 0).all() and (m <= 1).all()
    np.testing.assert_allclose(eps.cpu().numpy(), np.abs(m[..., 0]), rtol=1e-6)     # one query row: eps = m
    idx, count = buf.idx.cpu().numpy(), buf.count.cpu().numpy()
    G = w.group
    for b, g in ((0, 0), (7, 3), (15, 7)):
        hs = slice(g * G, (g + 1) * G)
        qd, kk, vv = f32(q_dec[b:b + 1, hs]), f32(t["k"][b:b + 1, g:g + 1]), f32(t["v"][b:b + 1, g:g + 1])
        ro, rl = oracle.decode_attention(qd, kk, vv)
        _close_rows(out_f[b:b + 1, hs], ro, f"full cache unit ({b},{g})")
        np.testing.assert_allclose(lse_f[b:b + 1, hs], rl, atol=1e-4, rtol=0)
        n = int(count[b, g])
        ro, rl = oracle.decode_attention(qd, f32(buf.k_out[b:b + 1, g:g + 1]), f32(buf.v_out[b:b + 1, g:g + 1]),
                                         count[b:b + 1, g:g + 1])
        _close_rows(out_c[b:b + 1, hs], ro, f"compact cache unit ({b},{g})")
        np.testing.assert_allclose(lse_c[b:b + 1, hs], rl, atol=1e-4, rtol=0)
        rm = oracle.discarded_mass(qd, kk, idx[b:b + 1, g:g + 1], count[b:b + 1, g:g + 1])
        np.testing.assert_allclose(m[b:b + 1, hs], rm, atol=5e-5, rtol=1e-3)
