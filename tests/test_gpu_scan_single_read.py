"""GPU parity of the single-read scan (the persistent kernel behind ckv_window_scores that reads K once),
forced with CKV_FLAG_SCAN_SINGLE_READ on shapes chosen to reach each of its code paths, against the CPU
oracle and against the two-kernel scan on the same tensors."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import assert_scores_close, f32, params_of

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(name, Bz, Hq, Hkv, d, T, W, **kw):
    return wl.Workload(name, "bf16", Bz, Hq, Hkv, d, T, W, wl.POOL_AVG, 7, max(W + 8, min(T, W + T // 8)), 2,
                       seed=300 + T + W + Hq, **kw)


# With 32 workgroups (128 waves) per XCD, a wave takes ceil(ceil(T / 32) / 128) key tiles of a unit.
CASES = [
    _case("sr_short_gqa4", 2, 8, 2, 128, 1000, 32),                      # one tile per wave: masked path only
    _case("sr_units_lt_xcds", 1, 8, 2, 128, 20011, 32, pareto_frac=0.05),  # 5 tiles per wave: one round + left-over; idle XCDs
    _case("sr_full_capacity", 3, 12, 3, 128, 32768, 32, sink_scale=8.0),  # 8 tiles per wave, 9 units: two units on one XCD
    _case("sr_beyond_capacity", 1, 4, 1, 128, 45000, 32),                # 11 tiles per wave: three fetched again
    _case("sr_mha", 10, 1, 1, 128, 17000, 32),                           # one query tile, one phase
    _case("sr_gqa2", 5, 4, 2, 128, 16500, 32, needles=4),                # two tiles, two phases of one
    _case("sr_gqa3", 3, 9, 3, 128, 18000, 20),                           # three phases, ragged window
    _case("sr_w64_gqa2", 2, 8, 4, 128, 24000, 64, head_key_scale=True),  # two tiles per head, two heads
    _case("sr_w48_mha", 9, 1, 1, 128, 16400, 48),                        # padded second tile
    _case("sr_d64", 4, 8, 2, 64, 33000, 32),                             # 128-byte rows, 9 tiles per wave
    _case("sr_tiny", 1, 4, 1, 128, 40, 8),
    _case("sr_all_window", 1, 2, 1, 128, 32, 32),                        # P = 0
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_single_read_scan_matches_oracle(w):
    print(f"case {w.name}", flush=True)
    layer = wl.make_layer(w, 0, DEV)
    q, k, v = layer["q"], layer["k"], layer["v"]
    p1 = params_of(w, q, k, v, flags=B.FLAG_SCAN_SINGLE_READ)
    buf = B.LayerBuffers(p1, DEV)
    buf.scores.fill_(float("nan"))
    B.ckv_window_scores(p1, q, k, None, None, buf.scores, None, buf.workspace)
    torch.cuda.synchronize()
    off = B.ckv_scan_status_offset(p1)
    assert off >= 0 and off % 4 == 0
    assert int(buf.workspace.view(torch.uint8)[off:off + 4].view(torch.int32).item()) == 0, "a bounded wait expired"
    got = buf.scores.cpu().numpy()
    ref = oracle.window_scores(f32(q), f32(k))
    assert_scores_close(got, ref, "single-read scores")
    np.testing.assert_allclose(got.astype(np.float64).sum(-1), w.seq_len, rtol=2e-4)   # Eq. 4 remark
    # a second call on the same workspace (synchronisation words are re-initialised per call): bit-stable
    again = torch.full_like(buf.scores, float("nan"))
    B.ckv_window_scores(p1, q, k, None, None, again, None, buf.workspace)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(again.cpu().numpy(), got)
    # the two-kernel scan computes the same thing
    p2 = params_of(w, q, k, v, flags=B.FLAG_SCAN_TWO_KERNELS)
    two = torch.full_like(buf.scores, float("nan"))
    B.ckv_window_scores(p2, q, k, None, None, two, None, buf.workspace)
    torch.cuda.synchronize()
    assert_scores_close(two.cpu().numpy(), ref, "two-kernel scores")
