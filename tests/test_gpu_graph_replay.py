"""The library's calls only launch kernels (no allocation, no memset, no synchronisation), so a caller may
capture them into a HIP graph. One layer of the retention path and one decoding step are captured once and
replayed several times, with eager work and synchronisations in between; every replay must reproduce the
eager result bit for bit."""
import pytest
import torch

from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import params_of

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _outputs(buf, extra=()):
    return [t.clone() for t in (buf.utility, buf.budget, buf.tau, buf.idx, buf.count, buf.k_out, buf.v_out, *extra)]


@pytest.mark.parametrize("long_prefix", [False, True], ids=["register_select", "split_select"])
def test_retention_layer_and_decode_step_replay_from_a_graph(long_prefix):
    T = 70000 if long_prefix else 6000          # beyond 32768 prefix positions the selection takes six launches
    w = wl.Workload("graph", "bf16", 1, 8, 2, 128, T, 32, wl.POOL_AVG, 7, 400, 2, seed=77, pareto_frac=0.05, shares=True)
    layers = [wl.make_layer(w, l, DEV) for l in range(2)]
    tabs = wl.make_tables(w, DEV)
    q = torch.empty_like(layers[0]["q"])
    k = torch.empty_like(layers[0]["k"])
    v = torch.empty_like(layers[0]["v"])
    p = params_of(w, q, k, v)
    buf = B.LayerBuffers(p, DEV)
    q_dec = wl.make_decode_queries(w, 0, 1, DEV)
    out = torch.empty(w.batch, w.n_q_heads, 1, w.head_dim, device=DEV)
    lse = torch.empty(w.batch, w.n_q_heads, 1, device=DEV)
    ws = torch.empty(max(B.ckv_decode_workspace_bytes(p, 1, w.cap), 256), dtype=torch.uint8, device=DEV)

    def step():
        B.retention_layer(p, q, k, v, tabs, buf, fused_utility=True)
        B.ckv_decode_attention(p, q_dec, buf.k_out, buf.v_out, buf.count, out, lse, ws)

    def load(l):   # the graph reads its inputs from fixed buffers, as a serving loop would
        q.copy_(layers[l]["q"]); k.copy_(layers[l]["k"]); v.copy_(layers[l]["v"])
        buf.idx.fill_(-1); buf.k_out.zero_(); buf.v_out.zero_()

    eager = []
    for l in range(2):
        load(l)
        step()
        torch.cuda.synchronize()
        eager.append(_outputs(buf, (out, lse)))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        l = rep % 2
        load(l)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(_outputs(buf, (out, lse)), eager[l]):
            assert torch.equal(got, ref), f"replay {rep} differs from the eager run of layer {l}"
        (buf.utility.sum() + buf.k_out.float().sum()).item()   # eager library work between the replays
