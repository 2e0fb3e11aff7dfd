"""CPU oracle of CompilerKV's prefill-end retention step (paper Sec. 4, Alg. 1).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and by the CPU-baseline
leg of ``bench.py``. The product path (the HIP library and its binding) never imports this package,
and this package imports nothing from the product.

The arithmetic lives in ``ckv_oracle.c`` (plain C, fp64); this module compiles it with gcc on first
use, loads it with ctypes and exposes numpy-in / numpy-out functions. Inputs that are stored as bf16
on the device are passed here as float32 arrays holding exactly the same values.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "ckv_oracle.c"
_LIB = _HERE / "libckv_oracle.so"
_lib = None

POOL_NONE, POOL_AVG, POOL_MAX = 0, 1, 2
EPS_VALUE_NORM = 1e-6


def build(force: bool = False) -> Path:
    """Compile ckv_oracle.c into libckv_oracle.so next to it (gcc -O2 -fopenmp)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               str(_SRC), "-o", str(tmp), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i, d, p = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        lib.ckv_oracle_window_scores.argtypes = [i, i, i, i, i, i, d, p, p, p, p]
        lib.ckv_oracle_window_scores.restype = i
        lib.ckv_oracle_value_norm_ratio.argtypes = [i, i, i, i, d, p, p]
        lib.ckv_oracle_value_norm_ratio.restype = i
        lib.ckv_oracle_pool.argtypes = [i, i, i, i, p, p]
        lib.ckv_oracle_pool.restype = i
        lib.ckv_oracle_utility.argtypes = [i, i, i, i, i, i, i, p, p, p, p]
        lib.ckv_oracle_utility.restype = i
        lib.ckv_oracle_budgets.argtypes = [i, i, i, i, p, p]
        lib.ckv_oracle_budgets.restype = i
        lib.ckv_oracle_tau.argtypes = [p, i, i, i, i]
        lib.ckv_oracle_tau.restype = ctypes.c_float
        lib.ckv_oracle_select.argtypes = [i, i, i, i, i, p, p, p, p, p]
        lib.ckv_oracle_select.restype = i
        lib.ckv_oracle_gather.argtypes = [i, i, i, ctypes.c_size_t, p, p, p, p]
        lib.ckv_oracle_gather.restype = i
        lib.ckv_oracle_threads.argtypes = []
        lib.ckv_oracle_threads.restype = i
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def threads() -> int:
    return int(_load().ckv_oracle_threads())


def window_scores(q, k, scale=None, return_lse=False):
    """q [Bz,Hq,W,d], k [Bz,Hkv,T,d] float32 -> scores [Bz,Hq,T] float64 (and LSE [Bz,Hq,W])."""
    q, k = _f32(q), _f32(k)
    Bz, Hq, W, d = q.shape
    Bk, Hkv, T, dk = k.shape
    if Bk != Bz or dk != d:
        raise ValueError("q and k disagree on batch or head_dim")
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(float(d))
    scores = np.empty((Bz, Hq, T), dtype=np.float64)
    lse = np.empty((Bz, Hq, W), dtype=np.float64) if return_lse else None
    _check(_load().ckv_oracle_window_scores(Bz, Hq, Hkv, d, T, W, float(scale), _ptr(q), _ptr(k),
                                            _ptr(scores), _ptr(lse)), "window_scores")
    return (scores, lse) if return_lse else scores


def value_norm_ratio(v, eps=EPS_VALUE_NORM):
    """v [Bz,Hkv,T,d] float32 -> rho [Bz,Hkv,T] float64."""
    v = _f32(v)
    Bz, Hkv, T, d = v.shape
    rho = np.empty((Bz, Hkv, T), dtype=np.float64)
    _check(_load().ckv_oracle_value_norm_ratio(Bz, Hkv, T, d, float(eps), _ptr(v), _ptr(rho)),
           "value_norm_ratio")
    return rho


def pool(x, mode, kernel):
    """x [..., n] float64 -> same shape, pooled along the last axis."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    n = x.shape[-1]
    rows = int(np.prod(x.shape[:-1], dtype=np.int64)) if x.ndim > 1 else 1
    y = np.empty_like(x)
    _check(_load().ckv_oracle_pool(rows, n, int(mode), int(kernel), _ptr(x), _ptr(y)), "pool")
    return y


def utility(scores, W, n_kv_heads, mode, kernel, w_head_row, rho=None):
    """scores [Bz,Hq,T] float64 (+ rho [Bz,Hkv,T]) -> utility [Bz,Hkv,P] float32."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    Bz, Hq, T = scores.shape
    Hkv = int(n_kv_heads)
    w = _f32(w_head_row, (Hq,))
    if rho is not None:
        rho = np.ascontiguousarray(rho, dtype=np.float64)
        if rho.shape != (Bz, Hkv, T):
            raise ValueError("rho shape")
    out = np.empty((Bz, Hkv, T - W), dtype=np.float32)
    _check(_load().ckv_oracle_utility(Bz, Hq, Hkv, T, int(W), int(mode), int(kernel), _ptr(scores),
                                      _ptr(rho), _ptr(w), _ptr(out)), "utility")
    return out


def budgets(n_kv_heads, T, W, B, share_row=None):
    """Per-KV-head budgets of one layer -> int32 [Hkv]."""
    share = None if share_row is None else _f32(share_row, (n_kv_heads,))
    out = np.empty((n_kv_heads,), dtype=np.int32)
    _check(_load().ckv_oracle_budgets(int(n_kv_heads), int(T), int(W), int(B), _ptr(share), _ptr(out)),
           "budgets")
    return out


def tau(gate_layer, b_ent, b_ppl):
    """gate_layer [n_ent,n_ppl] float32 or None -> python float (exact fp32 value)."""
    if gate_layer is None:
        return 0.0
    g = _f32(gate_layer)
    return float(_load().ckv_oracle_tau(_ptr(g), g.shape[0], g.shape[1], int(b_ent), int(b_ppl)))


def select(utility_, tau_, budget, W, cap):
    """utility [Bz,Hkv,P] f32, tau [Bz] f32, budget [Bz,Hkv] i32 -> idx [Bz,Hkv,cap] (-1 padded), count."""
    u = _f32(utility_)
    Bz, Hkv, P = u.shape
    T = P + int(W)
    t = _f32(tau_, (Bz,))
    b = np.ascontiguousarray(budget, dtype=np.int32)
    if b.shape != (Bz, Hkv):
        raise ValueError("budget shape")
    idx = np.full((Bz, Hkv, int(cap)), -1, dtype=np.int32)
    count = np.empty((Bz, Hkv), dtype=np.int32)
    _check(_load().ckv_oracle_select(Bz, Hkv, T, int(W), int(cap), _ptr(u), _ptr(t), _ptr(b), _ptr(idx),
                                     _ptr(count)), "select")
    return idx, count


def gather(src, idx, count):
    """src [Bz,Hkv,T,...] any dtype, idx [Bz,Hkv,cap], count [Bz,Hkv] -> [Bz,Hkv,cap,...] (zeros beyond count)."""
    src = np.ascontiguousarray(src)
    Bz, Hkv, T = src.shape[:3]
    row_bytes = int(np.prod(src.shape[3:], dtype=np.int64)) * src.dtype.itemsize
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    count = np.ascontiguousarray(count, dtype=np.int32)
    cap = idx.shape[2]
    dst = np.zeros((Bz, Hkv, cap) + src.shape[3:], dtype=src.dtype)
    _check(_load().ckv_oracle_gather(Bz * Hkv, T, cap, row_bytes, _ptr(src), _ptr(idx), _ptr(count),
                                     _ptr(dst)), "gather")
    return dst


def retention_layer(q, k, v_bits, v=None, *, W, mode, kernel, B, cap, w_head_row, share_row=None,
                    gate_layer=None, risk_bins=None, value_norm=False, scale=None, k_bits=None):
    """The whole per-layer chain in Alg. 1's order. Returns a dict of every intermediate.

    q, k, v: float32 images of the stored tensors; k_bits / v_bits: the stored tensors' raw arrays
    (any dtype) for the byte-exact gather (k_bits defaults to k, v_bits may be None to skip V).
    """
    q, k = _f32(q), _f32(k)
    Bz, Hq = q.shape[:2]
    Hkv, T = k.shape[1], k.shape[2]
    s, lse = window_scores(q, k, scale, return_lse=True)
    rho = value_norm_ratio(v) if value_norm else None
    u = utility(s, W, Hkv, mode, kernel, w_head_row, rho)
    bud = np.tile(budgets(Hkv, T, W, B, share_row), (Bz, 1)).astype(np.int32)
    if gate_layer is None:
        tau_b = np.zeros((Bz,), dtype=np.float32)
    else:
        tau_b = np.array([tau(gate_layer, risk_bins[b][0], risk_bins[b][1]) for b in range(Bz)],
                         dtype=np.float32)
    idx, count = select(u, tau_b, bud, W, cap)
    out = dict(scores=s, lse=lse, rho=rho, utility=u, budget=bud, tau=tau_b, idx=idx, count=count)
    out["k_out"] = gather(k if k_bits is None else k_bits, idx, count)
    if v_bits is not None:
        out["v_out"] = gather(v_bits, idx, count)
    return out


# ---------------------------------------------------------------------------------------------------
# Layer-shared mode: Alg. 1 as printed -- one window mass alpha per prompt (the mean over all layers and
# heads, steps (A)), the structural risk coordinate, and per layer one utility vector and one index set
# shared by all heads (stages (B)-(D)). Plain numpy in float64, one statement per step of the listing.
# ---------------------------------------------------------------------------------------------------
def alpha_mean(scores_per_layer):
    """Per-head window masses of every layer, each [Bz,Hq,T] (already scaled by T/W) -> alpha [Bz,T]:
    alpha = (T/|Omega|) sum_j Abar[j,:] with Abar the mean of A over layers and heads (Eq. 4)."""
    stack = np.stack([np.asarray(s, dtype=np.float64) for s in scores_per_layer])   # [L,Bz,Hq,T]
    return stack.mean(axis=(0, 2))


def risk_struct(alpha):
    """alpha [Bz,T] -> structural risk [Bz]: entropy (natural log) of A' = alpha / ||alpha||_1 (Alg. 1 (A),
    Eq. 7); terms with A'_t = 0 contribute 0."""
    a = np.asarray(alpha, dtype=np.float64)
    p = a / a.sum(axis=-1, keepdims=True)
    terms = np.where(p > 0, p * np.log(np.where(p > 0, p, 1.0)), 0.0)
    return -terms.sum(axis=-1)


def discretize(value, edges):
    """Bin index of each value for ascending bin edges e_0 < e_1 < ...: the number of edges <= value
    (so n edges make n + 1 bins; the paper leaves the edges to the table's compiler)."""
    v = np.atleast_1d(np.asarray(value, dtype=np.float64))
    e = np.asarray(edges, dtype=np.float64)
    return np.array([int((e <= x).sum()) for x in v], dtype=np.int32)


def shared_utility(alpha, rho, w_head_row, W):
    """alpha [Bz,T], rho [Bz,Hkv,T], w_head_row [Hq] -> u_hat [Bz,P] float32 (Alg. 1 stages (B)-(C)):
    u^(h) = alpha * rho^(kv head of h); u_hat = max over ALL query heads of fp32(W_head[h] * u^(h))."""
    a = np.asarray(alpha, dtype=np.float64)
    r = np.asarray(rho, dtype=np.float64)
    w = np.asarray(w_head_row, dtype=np.float32)
    Bz, T = a.shape
    Hkv, Hq = r.shape[1], w.shape[0]
    G = Hq // Hkv
    P = T - int(W)
    best = np.full((Bz, P), -np.inf, dtype=np.float32)
    for h in range(Hq):
        u_h = a[:, :P] * r[:, h // G, :P]
        best = np.maximum(best, (np.float64(w[h]) * u_h).astype(np.float32))
    return best


def gather_shared(src, idx, count):
    """src [Bz,Hkv,T,...], idx [Bz,cap], count [Bz] -> [Bz,Hkv,cap,...]: every head of a layer keeps the
    same positions (Alg. 1: S^(l) is shared across heads within layer l)."""
    src = np.ascontiguousarray(src)
    Bz, Hkv = src.shape[:2]
    return gather(src, np.repeat(np.asarray(idx, np.int32)[:, None, :], Hkv, axis=1),
                  np.repeat(np.asarray(count, np.int32)[:, None], Hkv, axis=1))


def layer_shared_layer(alpha, k_bits, v_bits, v, *, W, B_layer, cap, w_head_row, gate_layer=None, risk_bins=None):
    """Stages (B)-(D) of Alg. 1 for one layer given the prompt's alpha: rho, u_hat, tau, the shared index
    set (window forced in, as in the per-head mode) and the gathered K/V."""
    a = np.asarray(alpha, dtype=np.float64)
    Bz = a.shape[0]
    rho = value_norm_ratio(v)
    u = shared_utility(a, rho, w_head_row, W)
    if gate_layer is None:
        tau_b = np.zeros((Bz,), dtype=np.float32)
    else:
        tau_b = np.array([tau(gate_layer, risk_bins[b][0], risk_bins[b][1]) for b in range(Bz)], dtype=np.float32)
    bud = np.full((Bz, 1), int(B_layer), dtype=np.int32)
    idx, count = select(u[:, None, :], tau_b, bud, W, cap)
    idx, count = idx[:, 0], count[:, 0]
    return dict(rho=rho, utility=u, tau=tau_b, idx=idx, count=count,
                k_out=gather_shared(k_bits, idx, count), v_out=gather_shared(v_bits, idx, count))


def map_table_depth(table, n_layers_dst):
    """Rows of a table compiled on L_src layers ([L_src, ...]) -> [L_dst, ...] for a model of another depth
    (App. "Model choice and cross-architecture applicability": a monotonic depth mapping, relative-depth
    interpolation): target layer l sits at relative depth l / (L_dst - 1), i.e. at source coordinate
    x = l (L_src - 1) / (L_dst - 1), and takes the linear interpolation of the two neighbouring source rows
    (row 0 for a one-layer target)."""
    t = np.asarray(table, dtype=np.float64)
    L_src, L_dst = t.shape[0], int(n_layers_dst)
    out = np.empty((L_dst,) + t.shape[1:], dtype=np.float64)
    for l in range(L_dst):
        x = 0.0 if L_dst == 1 else l * (L_src - 1) / (L_dst - 1)
        i = min(int(np.floor(x)), L_src - 1)
        j = min(i + 1, L_src - 1)
        f = x - i
        out[l] = (1.0 - f) * t[i] + f * t[j]
    return out


# ---------------------------------------------------------------------------------------------------
# Decode-side consumer (Proposition 1 and its proof in App. A): a decoding query attends over the
# retained set only; the discarded mass m_t of its full attention row measures what compression lost.
# Plain numpy in float64, rows written out explicitly.
# ---------------------------------------------------------------------------------------------------
def _logits(q_dec, keys, scale):
    """q_dec [Bz,Hq,Nq,d], keys [Bz,Hkv,R,d] -> scaled logits [Bz,Hq,Nq,R] (query head h reads KV head h // G)."""
    q = np.asarray(q_dec, dtype=np.float64)
    k = np.asarray(keys, dtype=np.float64)
    G = q.shape[1] // k.shape[1]
    s = (1.0 / np.sqrt(q.shape[-1])) if scale is None else float(scale)
    return s * np.einsum("bhqd,bhrd->bhqr", q, np.repeat(k, G, axis=1))


def decode_attention(q_dec, keys, values, count=None, scale=None):
    """Attention of decoding queries (positions after the prompt: every row is visible) over a ragged KV
    set: keys/values [Bz,Hkv,R,d] of which the first count[b,g] rows are valid (all R if count is None).
    Returns (out [Bz,Hq,Nq,d], lse [Bz,Hq,Nq]) with lse = log sum_j exp z_j over the valid rows -- the
    compressed row of Proposition 1, p~ = p restricted to S and renormalised, applied to V."""
    z = _logits(q_dec, keys, scale)
    v = np.asarray(values, dtype=np.float64)
    Bz, Hq, Nq, R = z.shape
    G = Hq // v.shape[1]
    out = np.zeros((Bz, Hq, Nq, v.shape[-1]))
    lse = np.zeros((Bz, Hq, Nq))
    for b in range(Bz):
        for h in range(Hq):
            n = R if count is None else int(count[b][h // G])
            for i in range(Nq):
                row = z[b, h, i, :n]
                top = row.max()
                e = np.exp(row - top)
                lse[b, h, i] = top + np.log(e.sum())
                out[b, h, i] = (e / e.sum()) @ v[b, h // G, :n]
    return out, lse


def attention_rows(q_dec, keys, idx=None, count=None, scale=None):
    """Full attention rows p [Bz,Hq,Nq,T] of decoding queries over all T keys and, if idx/count
    [Bz,Hkv,cap]/[Bz,Hkv] name a retained set S per KV head, the compressed rows p~ (zero outside S,
    renormalised over S; Proposition 1)."""
    z = _logits(q_dec, keys, scale)
    p = np.exp(z - z.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    if idx is None:
        return p
    Bz, Hq, Nq, T = p.shape
    G = Hq // np.asarray(keys).shape[1]
    keep = np.zeros((Bz, Hq, 1, T), dtype=bool)
    for b in range(Bz):
        for h in range(Hq):
            keep[b, h, 0, np.asarray(idx[b][h // G][: int(count[b][h // G])], dtype=np.int64)] = True
    kept = np.where(keep, p, 0.0)
    return p, kept / kept.sum(-1, keepdims=True)


def discarded_mass(q_dec, keys, idx, count, scale=None):
    """m [Bz,Hq,Nq]: the mass of each full attention row outside the retained set, summed term by term."""
    p = attention_rows(q_dec, keys, scale=scale)
    Bz, Hq, Nq, T = p.shape
    G = Hq // np.asarray(keys).shape[1]
    m = np.zeros((Bz, Hq, Nq))
    for b in range(Bz):
        for h in range(Hq):
            out = np.ones(T, dtype=bool)
            out[np.asarray(idx[b][h // G][: int(count[b][h // G])], dtype=np.int64)] = False
            m[b, h] = p[b, h][:, out].sum(-1)
    return m


def tail_eps(mass):
    """eps_tail [Bz,Hq] = sqrt(mean over the query rows of m^2) (Proposition 1)."""
    m = np.asarray(mass, dtype=np.float64)
    return np.sqrt((m * m).mean(-1))
