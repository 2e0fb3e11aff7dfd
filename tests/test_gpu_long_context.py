"""Contexts of one and a half and two million tokens (the scan's 32-bit offsets, the selection split over
hundreds of workgroups, the streaming selection for a prefix that is no multiple of four), through both
call sequences, every element against the oracle (8-13 s of oracle time per case on 16 cores)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import assert_index_sets_match, assert_scores_close, bits, params_of, run_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda"

CASES = [
    # P = 2^21: fused utility pass, 256 selection slices per unit
    wl.Workload("long_2m", "bf16", 1, 4, 1, 128, 2 ** 21 + 32, 32, wl.POOL_AVG, 7, 4096, 2, seed=4242, head_key_scale=True,
                shares=True, needles=8),
    # ragged everything: P % 4 = 3 (the two unfused steps, streaming selection), two tiles per head
    wl.Workload("long_1m5_ragged", "bf16", 1, 6, 2, 128, 1500007, 64, wl.POOL_MAX, 5, 4096, 2, seed=4243, sink_scale=8.0,
                shares=True, needles=8),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_long_context_chain_matches_oracle(w):
    print(f"case {w.name}", flush=True)
    t, tabs = wl.make_layer(w, 0, DEV), wl.make_tables(w, DEV)
    q, k, v = t["q"], t["k"], t["v"]
    ref = run_oracle(w, t, tabs, layer=0)
    p = params_of(w, q, k, v)
    for fused in (False, True):
        print(f"  fused={fused}", flush=True)
        buf = B.LayerBuffers(p, DEV)
        buf.scores.fill_(float("nan"))
        buf.utility.fill_(float("nan"))
        B.retention_layer(p, q, k, v, tabs, buf, fused_utility=fused)
        torch.cuda.synchronize()
        if not fused:
            s = buf.scores.cpu().numpy()
            assert_scores_close(s, ref["scores"])
            np.testing.assert_allclose(s.astype(np.float64).sum(-1), w.seq_len, rtol=2e-4)   # Eq. 4 remark
        gu = buf.utility.cpu().numpy()
        assert_scores_close(gu, ref["utility"].astype(np.float64), "utility")
        np.testing.assert_array_equal(buf.budget.cpu().numpy(), ref["budget"])
        gi, gc = buf.idx.cpu().numpy(), buf.count.cpu().numpy()
        assert_index_sets_match(gi, gc, ref["idx"], ref["count"], ref["utility"], ref["tau"], ref["budget"], w.window)
        oi, oc = oracle.select(gu, buf.tau.cpu().numpy(), buf.budget.cpu().numpy(), w.window, w.cap)
        np.testing.assert_array_equal(gc, oc)
        np.testing.assert_array_equal(gi, oi)
        np.testing.assert_array_equal(bits(buf.k_out), oracle.gather(bits(k), gi, gc))
        np.testing.assert_array_equal(bits(buf.v_out), oracle.gather(bits(v), gi, gc))
        for g in range(w.n_kv_heads):   # the planted keys are kept
            assert set(t["needle_pos"][0, g].tolist()) <= set(gi[0, g, : gc[0, g]].tolist())
