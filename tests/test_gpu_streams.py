"""Calls for different layers share nothing but their read-only inputs (each layer has its outputs and its
workspace), so a caller may queue them on different HIP streams and let them overlap, as the benchmark does.
Several layers are run one after another on one stream, then dealt to two and to three streams (default
priority); every output of every layer must come out bit for bit the same. Shapes: one whose selection is a
single launch and one with the six-launch selection of long prefixes, value norm on in one of them."""
import pytest
import torch

from paper_2602_08686_amd import binding as B
from paper_2602_08686_amd import workloads as wl
from parity_util import params_of

pytestmark = pytest.mark.gpu
DEV = "cuda"
N_LAYERS = 6


def _outputs(buf):
    return [t.clone() for t in (buf.utility, buf.budget, buf.tau, buf.idx, buf.count, buf.k_out, buf.v_out)]


@pytest.mark.parametrize("T,value_norm", [(9000, False), (40000, True)], ids=["register_select", "split_select_vnorm"])
def test_layers_on_several_streams_match_one_stream(T, value_norm):
    w = wl.Workload("streams", "bf16", 2, 8, 2, 128, T, 32, wl.POOL_MAX, 5, 300, N_LAYERS, seed=31, pareto_frac=0.05,
                    shares=True)
    print(f"case T={T} value_norm={value_norm}", flush=True)
    layers = [wl.make_layer(w, l, DEV) for l in range(N_LAYERS)]
    tabs = wl.make_tables(w, DEV)
    flags = B.FLAG_VALUE_NORM if value_norm else 0
    params = [params_of(w, layers[l]["q"], layers[l]["k"], layers[l]["v"], layer=l, flags=flags) for l in range(N_LAYERS)]
    bufs = [B.LayerBuffers(params[l], DEV) for l in range(N_LAYERS)]

    def run(streams):
        for b_ in bufs:
            b_.idx.fill_(-1); b_.k_out.zero_(); b_.v_out.zero_(); b_.utility.fill_(float("nan"))
        torch.cuda.synchronize()
        for rep in range(2):   # twice, so that a layer's kernels also overlap its own previous outputs' readers
            for l in range(N_LAYERS):
                t = layers[l]
                st = None if streams is None else streams[l % len(streams)]
                B.retention_layer(params[l], t["q"], t["k"], t["v"], tabs, bufs[l], stream=st, fused_utility=True)
        torch.cuda.synchronize()
        return [_outputs(b_) for b_ in bufs]

    serial = run(None)
    for n in (2, 3):
        got = run([torch.cuda.Stream() for _ in range(n)])
        for l in range(N_LAYERS):
            for a, b_ in zip(serial[l], got[l]):
                assert torch.equal(a, b_), f"layer {l}, {n} streams"
    assert all(torch.isfinite(o[0]).all() for o in serial)   # every utility was written
