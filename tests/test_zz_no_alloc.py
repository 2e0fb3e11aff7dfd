"""The entry point that allocates nothing (ckv_window_lse_static: the pass's row partials live in a device
array of the library) against ckv_window_lse on the same tensors, through the C ABI: two calls in a row,
the second on a smaller input, each bit-identical to the workspace form (same kernels, same arithmetic),
and the first also against the CPU oracle. Runs last in the suite (file name), and passes alone."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import f32, params_of

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _lse_pair(w, layer):
    t = wl.make_layer(w, layer, DEV)
    q, k, v = t["q"], t["k"], t["v"]
    p = params_of(w, q, k, v, layer=layer)
    assert 0 < B.ckv_window_lse_static_bytes(p) <= B.STATIC_SCRATCH_BYTES
    ws = torch.empty(B.ckv_workspace_bytes(p), dtype=torch.uint8, device=DEV)
    ref = torch.full((w.batch, w.n_q_heads, w.window), float("nan"), device=DEV)
    got = torch.full_like(ref, float("nan"))
    B.ckv_window_lse(p, q, k, ref, ws)
    before = torch.cuda.memory_allocated()
    B.ckv_window_lse_static(p, q, k, got)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return t, ref, got


def test_static_scratch_matches_workspace_form_twice_in_a_row():
    big = wl.C3.scaled(name="na_big", batch=3, seq_len=20000, n_layers=2)
    small = wl.C2.scaled(name="na_small", n_q_heads=6, n_kv_heads=2, seq_len=3000, window=20, n_layers=2)
    for w, layer in ((big, 1), (small, 0)):
        print(f"case {w.name}", flush=True)
        t, ref, got = _lse_pair(w, layer)
        assert torch.isfinite(got).all()
        assert torch.equal(got, ref)
        if w is big:
            _, want = oracle.window_scores(f32(t["q"]), f32(t["k"]), return_lse=True)
            np.testing.assert_allclose(got.cpu().numpy(), want, rtol=0, atol=2e-5 * max(1.0, float(np.abs(want).max())))
