"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the header
declares, sizes its workspace, and rejects bad arguments before anything would be launched."""
import ctypes
import pathlib
import re

import pytest
import torch

from paper_2602_08686_amd import binding as B

HEADER = pathlib.Path(__file__).resolve().parents[1] / "include" / "ckv.h"


def _good(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=4096, window=32,
                dtype=torch.bfloat16, pool=B.POOL_AVG, pool_kernel=7, budget=256, cap=512)
    base.update(kw)
    return B.make_params(**base)


def test_exports_match_header():
    lib = B.load()
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    declared = set(re.findall(r"\b(ckv_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layout_matches_header():
    # field order and count of ckv_params in the header vs. the ctypes mirror
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    body = re.search(r"typedef struct \{(.*?)\} ckv_params;", text, flags=re.S).group(1)
    names = re.findall(r"\b([a-z_]+)(?:\[3\])?;", body)
    assert names == [f[0] for f in B.CkvParams._fields_]
    assert ctypes.sizeof(B.CkvParams) == 40 + 72 + 20 + 4  # 10 x 4, 9 x 8, 5 x 4, tail padding


def test_status_strings():
    assert B.status_string(B.CKV_OK) == "ok"
    for s in range(1, 5):
        assert B.status_string(s)
    assert "unknown" in B.status_string(99)


def test_workspace_bytes_is_aligned_and_scales():
    a = B.ckv_workspace_bytes(_good())
    b = B.ckv_workspace_bytes(_good(batch=8))
    assert a > 0 and a % 256 == 0 and b > a
    assert B.ckv_workspace_bytes(_good(flags=B.FLAG_VALUE_NORM)) > a


@pytest.mark.parametrize("bad", [
    dict(n_q_heads=7),                 # Hq % Hkv
    dict(window=0), dict(window=5000),  # W outside [1, T]
    dict(pool_kernel=6),               # even kernel
    dict(pool=5),
    dict(budget=16),                   # B < W
    dict(cap=100),                     # cap below the largest possible per-head budget
    dict(layer=1, n_layers=1),
    dict(flags=16),                    # unknown flag
    dict(flags=8 | 4),                 # group masses exclude the single-read scan
    dict(softmax_scale=-1.0),
    dict(k_stride=(4096 * 128 * 2, 4096 * 128, 127)),   # row stride < head_dim / misaligned
    dict(q_stride=(8 * 32 * 128, 32 * 128 + 4, 128)),   # not 16-byte aligned
])
def test_invalid_params_are_rejected_on_the_host(bad):
    p = _good(**bad)
    assert B.ckv_workspace_bytes(p) == 0
    lib = B.load()
    dummy = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    st = lib.ckv_window_scores(ctypes.byref(p), dummy, dummy, None, None, dummy, None, dummy, 1 << 30, None)
    assert st == B.CKV_EINVAL
    st = lib.ckv_compact_kv(ctypes.byref(p), dummy, dummy, dummy, dummy, dummy, dummy, None)
    assert st == B.CKV_EINVAL


def test_unsupported_shapes():
    lib = B.load()
    dummy = ctypes.c_void_p(256)
    for kw in (dict(head_dim=96), dict(window=160, budget=256)):
        p = _good(**kw)
        st = lib.ckv_select_topk(ctypes.byref(p), dummy, dummy, dummy, dummy, dummy, None, 0, None)
        assert st == B.CKV_EUNSUPPORTED


def test_null_pointers_and_workspace_errors():
    lib = B.load()
    p = _good()
    dummy = ctypes.c_void_p(256)
    need = B.ckv_workspace_bytes(p)
    assert lib.ckv_window_scores(ctypes.byref(p), None, dummy, None, None, dummy, None, dummy, need, None) == B.CKV_EINVAL
    assert lib.ckv_window_scores(ctypes.byref(p), dummy, dummy, None, None, dummy, None, None, need, None) == B.CKV_EWORKSPACE
    assert lib.ckv_window_scores(ctypes.byref(p), dummy, dummy, None, None, dummy, None, dummy, need - 1, None) == B.CKV_EWORKSPACE
    assert lib.ckv_window_scores(ctypes.byref(p), dummy, dummy, None, None, dummy, None, ctypes.c_void_p(264), need, None) == B.CKV_EWORKSPACE
    pv = _good(flags=B.FLAG_VALUE_NORM)
    assert lib.ckv_window_scores(ctypes.byref(pv), dummy, dummy, None, None, dummy, None, dummy, 1 << 30, None) == B.CKV_EINVAL
    assert lib.ckv_apply_tables(ctypes.byref(p), dummy, None, None, None, None, 0, 0, None, dummy, dummy, dummy, None) == B.CKV_EINVAL
    assert lib.ckv_apply_tables(ctypes.byref(p), dummy, None, dummy, None, dummy, 20, 4, None, dummy, dummy, dummy, None) == B.CKV_EINVAL
    assert lib.ckv_select_topk(ctypes.byref(p), dummy, dummy, dummy, None, dummy, None, 0, None) == B.CKV_EINVAL
    assert lib.ckv_compact_kv(ctypes.byref(p), dummy, dummy, dummy, dummy, dummy, None, None) == B.CKV_EINVAL
    assert lib.ckv_window_scores(None, dummy, dummy, None, None, dummy, None, dummy, need, None) == B.CKV_EINVAL


def test_window_utility_and_scan_flags_are_validated_on_the_host():
    lib = B.load()
    p = _good()
    d = ctypes.c_void_p(256)
    need = B.ckv_workspace_bytes(p)
    wu = lambda prm, **kw: lib.ckv_window_utility(
        ctypes.byref(prm), kw.get("q", d), d, kw.get("v"), None, kw.get("w_head", d), None, kw.get("t_gate"),
        kw.get("n_ent", 0), 0, None, kw.get("scratch", d), kw.get("rho"), d, d, d, kw.get("ws", d),
        kw.get("ws_bytes", need), None)
    assert wu(p, q=None) == B.CKV_EINVAL
    assert wu(p, w_head=None) == B.CKV_EINVAL
    assert wu(p, scratch=None) == B.CKV_EINVAL
    assert wu(p, t_gate=d, n_ent=20) == B.CKV_EINVAL            # gate without risk bins
    assert wu(p, ws=None) == B.CKV_EWORKSPACE
    assert wu(p, ws_bytes=need - 1) == B.CKV_EWORKSPACE
    assert wu(_good(flags=B.FLAG_VALUE_NORM)) == B.CKV_EINVAL   # value norm without v / rho
    assert wu(_good(pool_kernel=6)) == B.CKV_EINVAL
    assert B.ckv_workspace_bytes(_good(flags=2)) == 0 and B.ckv_workspace_bytes(_good(flags=4)) == 0   # unknown flag bits


def test_layer_shared_entry_points_are_validated_on_the_host():
    lib = B.load()
    p = _good()
    ref = ctypes.byref
    d = ctypes.c_void_p(256)
    f = ctypes.c_float
    assert lib.ckv_alpha_accumulate(ref(p), None, f(0.5), d, None) == B.CKV_EINVAL
    assert lib.ckv_alpha_accumulate(ref(p), d, f(0.5), None, None) == B.CKV_EINVAL
    assert lib.ckv_alpha_accumulate(ref(p), d, f(float("nan")), d, None) == B.CKV_EINVAL
    assert lib.ckv_alpha_accumulate(None, d, f(0.5), d, None) == B.CKV_EINVAL
    assert lib.ckv_risk_struct(ref(p), None, None, 0, d, None, None) == B.CKV_EINVAL
    assert lib.ckv_risk_struct(ref(p), d, None, 0, None, None, None) == B.CKV_EINVAL
    assert lib.ckv_risk_struct(ref(p), d, None, -1, d, None, None) == B.CKV_EINVAL
    assert lib.ckv_risk_struct(ref(p), d, None, 19, d, d, None) == B.CKV_EINVAL      # bins asked for, no edges
    su = lambda **kw: lib.ckv_shared_utility(ref(p), kw.get("alpha", d), kw.get("rho", d), kw.get("w_head", d),
                                             kw.get("t_gate"), kw.get("n_ent", 0), kw.get("n_ppl", 0), kw.get("bins"),
                                             kw.get("util", d), kw.get("tau", d), None)
    for name in ("alpha", "rho", "w_head", "util", "tau"):
        assert su(**{name: None}) == B.CKV_EINVAL
    assert su(t_gate=d, n_ent=20, n_ppl=4) == B.CKV_EINVAL                          # gate without risk bins
    assert su(t_gate=d, n_ent=0, n_ppl=4, bins=d) == B.CKV_EINVAL
    args = [d] * 6
    for i in range(6):
        bad = list(args)
        bad[i] = None
        assert lib.ckv_compact_kv_shared(ref(p), *bad, None) == B.CKV_EINVAL
    assert lib.ckv_compact_kv_shared(ref(_good(window=0)), *args, None) == B.CKV_EINVAL


def test_decode_consumer_entry_points_are_validated_on_the_host():
    lib = B.load()
    p = _good()
    ref = ctypes.byref
    d = ctypes.c_void_p(256)
    rows = 20000
    need = B.ckv_decode_workspace_bytes(p, 1, rows)
    assert need > 0 and need % 256 == 0
    assert B.ckv_decode_workspace_bytes(p, 0, rows) == 0 and B.ckv_decode_workspace_bytes(p, 1, 0) == 0
    assert B.ckv_decode_workspace_bytes(p, 4, rows) >= need
    assert B.ckv_decode_workspace_bytes(p, 1, 544) == 0          # a short KV set is finished by one launch: no scratch
    good = (ctypes.c_int64 * 3)(8 * rows * 128, rows * 128, 128)
    st = lambda a: ctypes.cast(a, ctypes.c_void_p)
    da = lambda **kw: lib.ckv_decode_attention(
        ref(p), kw.get("q", d), kw.get("n_q", 1), kw.get("k", d), kw.get("v", d), st(kw.get("ks", good)),
        st(kw.get("vs", good)), kw.get("n_rows", rows), kw.get("count"), kw.get("out", d), kw.get("lse", d),
        kw.get("ws", d), kw.get("ws_bytes", need), None)
    for name in ("q", "k", "v", "out", "lse"):
        assert da(**{name: None}) == B.CKV_EINVAL
    assert da(q=ctypes.c_void_p(264)) == B.CKV_EINVAL                               # 16-byte alignment
    assert da(n_q=0) == B.CKV_EINVAL and da(n_rows=0) == B.CKV_EINVAL
    assert da(ks=(ctypes.c_int64 * 3)(8 * rows * 128, rows * 128, 64)) == B.CKV_EINVAL    # rows overlap
    assert da(vs=(ctypes.c_int64 * 3)(8 * rows * 128, rows * 128 + 4, 128)) == B.CKV_EINVAL  # not 16-byte pieces
    assert da(ks=(ctypes.c_int64 * 3)(-1, rows * 128, 128)) == B.CKV_EINVAL
    assert da(ws=None) == B.CKV_EWORKSPACE and da(ws_bytes=need - 256) == B.CKV_EWORKSPACE
    assert da(ws=ctypes.c_void_p(272)) == B.CKV_EWORKSPACE
    assert da(n_q=20000) == B.CKV_EUNSUPPORTED                                       # more query rows than one launch takes
    assert B.ckv_decode_workspace_bytes(p, 20000, rows) == 0
    dm = lambda **kw: lib.ckv_discarded_mass(ref(p), kw.get("n_q", 1), kw.get("lf", d), kw.get("lk", d),
                                             kw.get("mass", d), None, None)
    for name in ("lf", "lk", "mass"):
        assert dm(**{name: None}) == B.CKV_EINVAL
    assert dm(n_q=0) == B.CKV_EINVAL


def test_group_mass_flag_is_validated_on_the_host():
    lib = B.load()
    ref = ctypes.byref
    d = ctypes.c_void_p(256)
    p = _good(flags=B.FLAG_GROUP_MASS)
    need = B.ckv_workspace_bytes(p)
    assert need > 0
    # the calls that need per-head masses reject the flag
    assert lib.ckv_apply_tables(ref(p), d, None, d, None, None, 0, 0, None, d, d, d, None) == B.CKV_EINVAL
    assert lib.ckv_window_utility(ref(p), d, d, None, None, d, None, None, 0, 0, None, d, None, d, d, d, d, need,
                                  None) == B.CKV_EINVAL
    # shapes without the group-mass form: f32, W > 32, more than four heads per KV head
    for kw in (dict(dtype=torch.float32, head_dim=64), dict(window=64, budget=256), dict(n_q_heads=16, n_kv_heads=2)):
        q = _good(flags=B.FLAG_GROUP_MASS, **kw)
        n = B.ckv_workspace_bytes(q)
        assert n > 0
        assert lib.ckv_window_scores(ref(q), d, d, None, None, d, None, d, n, None) == B.CKV_EUNSUPPORTED


def test_depth_mapping_is_validated_on_the_host():
    lib = B.load()
    d = ctypes.c_void_p(256)
    assert lib.ckv_map_table_depth(None, 32, 8, d, 28, None) == B.CKV_EINVAL
    assert lib.ckv_map_table_depth(d, 32, 8, None, 28, None) == B.CKV_EINVAL
    for bad in ((0, 8, 28), (32, 0, 28), (32, 8, 0)):
        assert lib.ckv_map_table_depth(d, bad[0], bad[1], d, bad[2], None) == B.CKV_EINVAL
    assert lib.ckv_map_table_depth(d, 32, 1 << 20, d, 1 << 12, None) == B.CKV_EUNSUPPORTED


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        B.load(tmp_path / "libckv.so")


def test_static_scratch_rejects_shapes_beyond_its_array():
    lib = B.load()
    # 64 batch elements x 8 KV heads x 128 rows x 8 workgroups along the keys x 8 bytes > 4 MiB
    p = B.make_params(batch=64, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=1 << 20, window=32, dtype="bf16",
                      pool=B.POOL_AVG, pool_kernel=7, budget=512, cap=4096)
    need = B.ckv_window_lse_static_bytes(p)
    assert need > B.STATIC_SCRATCH_BYTES
    d = ctypes.c_void_p(256)
    assert lib.ckv_window_lse_static(ctypes.byref(p), d, d, d, None) == B.CKV_EWORKSPACE
