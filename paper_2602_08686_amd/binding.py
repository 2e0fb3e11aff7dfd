"""ctypes binding of libckv.so: the same four calls as ``include/ckv.h``, argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the retention path runs in
the library's kernels. There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libckv.so"
_lib = None

CKV_OK, CKV_EINVAL, CKV_EUNSUPPORTED, CKV_EWORKSPACE, CKV_EHIP = range(5)
CKV_F32, CKV_BF16 = 0, 1
POOL_NONE, POOL_AVG, POOL_MAX = 0, 1, 2
FLAG_VALUE_NORM = 1
FLAG_GROUP_MASS = 8         # ckv_window_scores writes per-KV-head sums [Bz,Hkv,T] (layer-shared mode)

EXPORTS = ("ckv_workspace_bytes", "ckv_window_lse", "ckv_window_lse_static_bytes", "ckv_window_lse_static", "ckv_window_scores", "ckv_window_utility", "ckv_apply_tables", "ckv_select_topk",
           "ckv_compact_kv", "ckv_alpha_accumulate", "ckv_risk_struct", "ckv_shared_utility", "ckv_compact_kv_shared",
           "ckv_decode_workspace_bytes", "ckv_decode_attention", "ckv_discarded_mass", "ckv_map_table_depth",
           "ckv_status_string")


class CkvParams(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("window", ctypes.c_int32),
        ("layer", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
        ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3), ("v_stride", ctypes.c_int64 * 3),
        ("pool", ctypes.c_int32), ("pool_kernel", ctypes.c_int32),
        ("budget_per_kv_head", ctypes.c_int32), ("cap", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


class CkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load(path: Optional[Path] = None):
    """Load libckv.so (once) and declare the signatures. Raises if the library has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = Path(path) if path else _LIB_PATH
    if not p.exists():
        raise FileNotFoundError(
            f"{p} is missing: build it with `python -m paper_2602_08686_amd.build` (hipcc, gfx950). "
            "There is no fallback path.")
    lib = ctypes.CDLL(str(p))
    vp, pp = ctypes.c_void_p, ctypes.POINTER(CkvParams)
    lib.ckv_workspace_bytes.argtypes = [pp]
    lib.ckv_workspace_bytes.restype = ctypes.c_size_t
    lib.ckv_window_scores.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.ckv_window_scores.restype = ctypes.c_int
    lib.ckv_window_lse.argtypes = [pp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.ckv_window_lse.restype = ctypes.c_int
    lib.ckv_window_lse_static_bytes.argtypes = [pp]
    lib.ckv_window_lse_static_bytes.restype = ctypes.c_size_t
    lib.ckv_window_lse_static.argtypes = [pp, vp, vp, vp, vp]
    lib.ckv_window_lse_static.restype = ctypes.c_int
    lib.ckv_window_utility.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp,
                                       vp, vp, ctypes.c_size_t, vp]
    lib.ckv_window_utility.restype = ctypes.c_int
    lib.ckv_apply_tables.argtypes = [pp, vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp]
    lib.ckv_apply_tables.restype = ctypes.c_int
    lib.ckv_select_topk.argtypes = [pp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.ckv_select_topk.restype = ctypes.c_int
    lib.ckv_compact_kv.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
    lib.ckv_compact_kv.restype = ctypes.c_int
    lib.ckv_alpha_accumulate.argtypes = [pp, vp, ctypes.c_float, vp, vp]
    lib.ckv_alpha_accumulate.restype = ctypes.c_int
    lib.ckv_risk_struct.argtypes = [pp, vp, vp, ctypes.c_int32, vp, vp, vp]
    lib.ckv_risk_struct.restype = ctypes.c_int
    lib.ckv_shared_utility.argtypes = [pp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp]
    lib.ckv_shared_utility.restype = ctypes.c_int
    lib.ckv_compact_kv_shared.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
    lib.ckv_compact_kv_shared.restype = ctypes.c_int
    lib.ckv_decode_workspace_bytes.argtypes = [pp, ctypes.c_int32, ctypes.c_int32]
    lib.ckv_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.ckv_decode_attention.argtypes = [pp, vp, ctypes.c_int32, vp, vp, vp, vp, ctypes.c_int32, vp, vp, vp, vp,
                                         ctypes.c_size_t, vp]
    lib.ckv_decode_attention.restype = ctypes.c_int
    lib.ckv_discarded_mass.argtypes = [pp, ctypes.c_int32, vp, vp, vp, vp, vp]
    lib.ckv_discarded_mass.restype = ctypes.c_int
    lib.ckv_map_table_depth.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp, ctypes.c_int32, vp]
    lib.ckv_map_table_depth.restype = ctypes.c_int
    lib.ckv_status_string.argtypes = [ctypes.c_int]
    lib.ckv_status_string.restype = ctypes.c_char_p
    if path is None:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().ckv_status_string(int(status)).decode()


def make_params(*, batch, n_q_heads, n_kv_heads, head_dim, seq_len, window, dtype, pool, pool_kernel,
                budget, cap, layer=0, n_layers=1, softmax_scale=0.0, flags=0,
                q_stride=None, k_stride=None, v_stride=None) -> CkvParams:
    """Fill a ckv_params; strides default to dense [Bz,H,rows,d] tensors."""
    p = CkvParams()
    p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim = batch, n_q_heads, n_kv_heads, head_dim
    p.seq_len, p.window, p.layer, p.n_layers = seq_len, window, layer, n_layers
    if isinstance(dtype, torch.dtype):
        dtype = {torch.bfloat16: "bf16", torch.float32: "f32"}.get(dtype)
    if dtype not in ("bf16", "f32"):
        raise ValueError("dtype must be float32 or bfloat16")
    p.dtype = CKV_BF16 if dtype == "bf16" else CKV_F32
    p.softmax_scale = softmax_scale
    dq = (n_q_heads * window * head_dim, window * head_dim, head_dim)
    dk = (n_kv_heads * seq_len * head_dim, seq_len * head_dim, head_dim)
    for name, val, dflt in (("q_stride", q_stride, dq), ("k_stride", k_stride, dk), ("v_stride", v_stride, dk)):
        arr = getattr(p, name)
        for i, s in enumerate(val if val is not None else dflt):
            arr[i] = int(s)
    p.pool, p.pool_kernel, p.budget_per_kv_head, p.cap, p.flags = pool, pool_kernel, budget, cap, flags
    return p


def params_for(q: torch.Tensor, k: torch.Tensor, v: Optional[torch.Tensor], *, pool, pool_kernel, budget,
               cap, layer=0, n_layers=1, softmax_scale=0.0, flags=0) -> CkvParams:
    """ckv_params describing the given tensors (any strides with a contiguous last axis)."""
    Bz, Hq, W, d = q.shape
    _, Hkv, T, _ = k.shape
    return make_params(batch=Bz, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, seq_len=T, window=W,
                       dtype=q.dtype, pool=pool, pool_kernel=pool_kernel, budget=budget, cap=cap,
                       layer=layer, n_layers=n_layers, softmax_scale=softmax_scale, flags=flags,
                       q_stride=q.stride()[:3], k_stride=k.stride()[:3],
                       v_stride=(v if v is not None else k).stride()[:3])


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != CKV_OK:
        raise CkvError(status, where)


def ckv_workspace_bytes(params: CkvParams) -> int:
    return int(load().ckv_workspace_bytes(ctypes.byref(params)))


def ckv_window_scores(params, q_win, k, v, lse, scores, vnorm_ratio, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().ckv_window_scores(ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(v), _ptr(lse),
                                    _ptr(scores), _ptr(vnorm_ratio), _ptr(workspace), nbytes,
                                    _stream(stream)), "ckv_window_scores")


def ckv_window_lse(params, q_win, k, lse, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().ckv_window_lse(ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(lse), _ptr(workspace),
                                 nbytes, _stream(stream)), "ckv_window_lse")


STATIC_SCRATCH_BYTES = 4 << 20


def ckv_window_lse_static_bytes(params: CkvParams) -> int:
    return int(load().ckv_window_lse_static_bytes(ctypes.byref(params)))


def ckv_window_lse_static(params, q_win, k, lse, stream=None):
    """ckv_window_lse without a workspace argument (the library's own device array holds the scratch)."""
    _check(load().ckv_window_lse_static(ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(lse), _stream(stream)),
           "ckv_window_lse_static")


def ckv_apply_tables(params, scores, vnorm_ratio, w_head, head_share, t_gate, n_ent, n_ppl, risk_bins,
                     utility, budget, tau, stream=None):
    _check(load().ckv_apply_tables(ctypes.byref(params), _ptr(scores), _ptr(vnorm_ratio), _ptr(w_head),
                                   _ptr(head_share), _ptr(t_gate), int(n_ent), int(n_ppl), _ptr(risk_bins),
                                   _ptr(utility), _ptr(budget), _ptr(tau), _stream(stream)),
           "ckv_apply_tables")


def ckv_window_utility(params, q_win, k, v, lse, w_head, head_share, t_gate, n_ent, n_ppl, risk_bins,
                       scores_scratch, vnorm_ratio, utility, budget, tau, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().ckv_window_utility(ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(v), _ptr(lse), _ptr(w_head),
                                     _ptr(head_share), _ptr(t_gate), int(n_ent), int(n_ppl), _ptr(risk_bins),
                                     _ptr(scores_scratch), _ptr(vnorm_ratio), _ptr(utility), _ptr(budget),
                                     _ptr(tau), _ptr(workspace), nbytes, _stream(stream)), "ckv_window_utility")


def ckv_select_topk(params, utility, budget, tau, idx, count, workspace=None, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().ckv_select_topk(ctypes.byref(params), _ptr(utility), _ptr(budget), _ptr(tau), _ptr(idx),
                                  _ptr(count), _ptr(workspace), nbytes, _stream(stream)), "ckv_select_topk")


def ckv_compact_kv(params, k, v, idx, count, k_out, v_out, stream=None):
    _check(load().ckv_compact_kv(ctypes.byref(params), _ptr(k), _ptr(v), _ptr(idx), _ptr(count),
                                 _ptr(k_out), _ptr(v_out), _stream(stream)), "ckv_compact_kv")


def ckv_alpha_accumulate(params, scores, weight, alpha, stream=None):
    _check(load().ckv_alpha_accumulate(ctypes.byref(params), _ptr(scores), float(weight), _ptr(alpha),
                                       _stream(stream)), "ckv_alpha_accumulate")


def ckv_risk_struct(params, alpha, ent_edges, risk, bins=None, stream=None):
    n = 0 if ent_edges is None else ent_edges.numel()
    _check(load().ckv_risk_struct(ctypes.byref(params), _ptr(alpha), _ptr(ent_edges), int(n), _ptr(risk),
                                  _ptr(bins), _stream(stream)), "ckv_risk_struct")


def ckv_shared_utility(params, alpha, vnorm_ratio, w_head, t_gate, n_ent, n_ppl, risk_bins, utility, tau,
                       stream=None):
    _check(load().ckv_shared_utility(ctypes.byref(params), _ptr(alpha), _ptr(vnorm_ratio), _ptr(w_head),
                                     _ptr(t_gate), int(n_ent), int(n_ppl), _ptr(risk_bins), _ptr(utility),
                                     _ptr(tau), _stream(stream)), "ckv_shared_utility")


def ckv_compact_kv_shared(params, k, v, idx, count, k_out, v_out, stream=None):
    _check(load().ckv_compact_kv_shared(ctypes.byref(params), _ptr(k), _ptr(v), _ptr(idx), _ptr(count),
                                        _ptr(k_out), _ptr(v_out), _stream(stream)), "ckv_compact_kv_shared")


def ckv_map_table_depth(table, mapped, stream=None):
    """table [L_src, ...] fp32 -> mapped [L_dst, ...] fp32 (same trailing shape), both contiguous."""
    row = table[0].numel()
    _check(load().ckv_map_table_depth(_ptr(table), int(table.shape[0]), int(row), _ptr(mapped), int(mapped.shape[0]),
                                      _stream(stream)), "ckv_map_table_depth")


def ckv_decode_workspace_bytes(params, n_q, n_rows) -> int:
    return int(load().ckv_decode_workspace_bytes(ctypes.byref(params), int(n_q), int(n_rows)))


def ckv_decode_attention(params, q_dec, k_rows, v_rows, count, out, lse, workspace, stream=None):
    """q_dec [Bz,Hq,n_q,d]; k_rows / v_rows [Bz,Hkv,n_rows,d] (any strides over the first three axes);
    count [Bz,Hkv] int32 or None."""
    n_q, n_rows = q_dec.shape[2], k_rows.shape[2]
    ks = (ctypes.c_int64 * 3)(*k_rows.stride()[:3])
    vs = (ctypes.c_int64 * 3)(*v_rows.stride()[:3])
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().ckv_decode_attention(ctypes.byref(params), _ptr(q_dec), int(n_q), _ptr(k_rows), _ptr(v_rows),
                                       ctypes.cast(ks, ctypes.c_void_p), ctypes.cast(vs, ctypes.c_void_p),
                                       int(n_rows), _ptr(count), _ptr(out), _ptr(lse), _ptr(workspace), nbytes,
                                       _stream(stream)), "ckv_decode_attention")


def ckv_discarded_mass(params, n_q, lse_full, lse_kept, mass, eps_tail=None, stream=None):
    _check(load().ckv_discarded_mass(ctypes.byref(params), int(n_q), _ptr(lse_full), _ptr(lse_kept), _ptr(mass),
                                     _ptr(eps_tail), _stream(stream)), "ckv_discarded_mass")


class LayerBuffers:
    """Device buffers for one layer's outputs and scratch, allocated once through PyTorch."""

    def __init__(self, params: CkvParams, device="cuda"):
        Bz, Hq, Hkv, T, W = params.batch, params.n_q_heads, params.n_kv_heads, params.seq_len, params.window
        d, cap = params.head_dim, params.cap
        dt = torch.bfloat16 if params.dtype == CKV_BF16 else torch.float32
        f32, i32 = torch.float32, torch.int32
        self.scores = torch.empty(Bz, Hq, T, dtype=f32, device=device)
        self.vnorm_ratio = (torch.empty(Bz, Hkv, T, dtype=f32, device=device)
                            if params.flags & FLAG_VALUE_NORM else None)
        self.utility = torch.empty(Bz, Hkv, T - W, dtype=f32, device=device)
        self.budget = torch.empty(Bz, Hkv, dtype=i32, device=device)
        self.tau = torch.empty(Bz, dtype=f32, device=device)
        self.idx = torch.full((Bz, Hkv, cap), -1, dtype=i32, device=device)
        self.count = torch.empty(Bz, Hkv, dtype=i32, device=device)
        self.k_out = torch.zeros(Bz, Hkv, cap, d, dtype=dt, device=device)
        self.v_out = torch.zeros(Bz, Hkv, cap, d, dtype=dt, device=device)
        self.workspace = torch.empty(max(ckv_workspace_bytes(params), 256), dtype=torch.uint8, device=device)


def retention_layer(params: CkvParams, q, k, v, tables: dict, buf: LayerBuffers, lse=None, stream=None,
                    fused_utility=False):
    """Queues the calls of one layer back-to-back on the stream; returns nothing (outputs in buf).
    fused_utility: ckv_window_utility in place of ckv_window_scores + ckv_apply_tables (buf.scores is
    then scratch)."""
    vv = v if params.flags & FLAG_VALUE_NORM else None
    if fused_utility:
        ckv_window_utility(params, q, k, vv, lse, tables["w_head"], tables.get("head_share"), tables.get("t_gate"),
                           tables.get("n_ent", 0), tables.get("n_ppl", 0), tables.get("risk_bins"), buf.scores,
                           buf.vnorm_ratio, buf.utility, buf.budget, buf.tau, buf.workspace, stream)
    else:
        ckv_window_scores(params, q, k, vv, lse, buf.scores, buf.vnorm_ratio, buf.workspace, stream)
        ckv_apply_tables(params, buf.scores, buf.vnorm_ratio, tables["w_head"], tables.get("head_share"),
                         tables.get("t_gate"), tables.get("n_ent", 0), tables.get("n_ppl", 0),
                         tables.get("risk_bins"), buf.utility, buf.budget, buf.tau, stream)
    ckv_select_topk(params, buf.utility, buf.budget, buf.tau, buf.idx, buf.count, buf.workspace, stream)
    ckv_compact_kv(params, k, v, buf.idx, buf.count, buf.k_out, buf.v_out, stream)
