#!/usr/bin/env python3
"""Benchmark of the prefill-end retention step (window scan + tables + select + gather) on one MI355X.

A step is one pass of the whole hot path over every layer of one synthetic prompt batch: for each
layer the C-ABI calls are queued back-to-back on a stream, every layer with its own K/V, output and
scratch buffers already resident in HBM. The layers of a step are dealt to `--streams` HIP streams in turn
(default 2; they are independent, so one layer's short kernels overlap the next layer's scan); the same
steps on a single stream are timed in the same run (`one_stream`). The headline value is algorithmic bytes moved per second
(what the method must read and write at least once, see `algorithmic_bytes`), to be read against
the 8 TB/s HBM peak; ms per layer is reported beside it. The same run also measures, with a few steps
each, the two other ways of calling the path (`modes`: LSE supplied by the caller, value-norm factor on),
and for short shapes the step replayed from a HIP graph (`roofline.graph_replay`).

Prints one JSON line. `--gpus N` with N > 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def algorithmic_bytes(w, kept_rows: int, value_norm: bool) -> int:
    """Bytes one layer must move at least once: K once, the Q window, V once only for the value-norm
    ratio, the gathered K and V rows read and written, the index lists and counts, the tables."""
    e = 2 if w.dtype == "bf16" else 4
    units = w.batch * w.n_kv_heads
    k_bytes = units * w.seq_len * w.head_dim * e
    q_bytes = w.batch * w.n_q_heads * w.window * w.head_dim * e
    v_bytes = k_bytes if value_norm else 0
    gather = 2 * 2 * kept_rows * w.head_dim * e
    idx = kept_rows * 4 + units * 4 * 2
    tables = (w.n_q_heads + w.n_kv_heads + 80) * 4
    return k_bytes + q_bytes + v_bytes + gather + idx + tables


def scan_bytes(w) -> int:
    """Algorithmic bytes of one scan launch (either pass): K once plus the Q window."""
    e = 2 if w.dtype == "bf16" else 4
    return (w.batch * w.n_kv_heads * w.seq_len + w.batch * w.n_q_heads * w.window) * w.head_dim * e


def scan_flops(w) -> float:
    return 2.0 * w.batch * w.n_q_heads * w.window * w.seq_len * w.head_dim


def kernel_source_digest() -> str:
    """sha256 over the HIP sources of the library (names and contents, in name order): what a counter summary under
    profiles/ is stamped with, so that a summary taken before a kernel changed is not passed off as current."""
    import hashlib

    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_08686_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` on the C3 workload as measured with rocprofv3 counters
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size): read from the committed summary of
    those runs, since counters cannot be collected from inside a timing run. None if not recorded, or
    if the summary's stamp (`sources=`) is not the digest of the kernel sources this run uses."""
    path = os.path.join(ROOT, "profiles", "pmc_hbm_traffic_c3.txt")
    current, found = False, None
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 2 and f[0] == "stamp" and f[1] == "sources=" + kernel_source_digest():
                current = True
            if len(f) == 4 and f[0] == "traffic" and f[1] == "kernel=" + kernel:
                found = int(f[2].split("=")[1]) + int(f[3].split("=")[1])
    except OSError:
        pass
    return found if current else None


def host_cpu() -> dict:
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"model": model, "nproc": os.cpu_count()}


def cpu_baseline(w, layer_t, tables, n_batch: int, value_norm: bool, single_thread: bool = False) -> dict:
    """Times the oracle (as it stands) on the first n_batch batch elements of layer 0."""
    import numpy as np
    import torch

    import oracle

    f32 = lambda t: t.detach().cpu().to(torch.float32).contiguous().numpy()
    raw = lambda t: (t.detach().cpu().contiguous().view(torch.int16).numpy()
                     if t.dtype == torch.bfloat16 else t.detach().cpu().contiguous().numpy())
    q, k, v = (layer_t[n][:n_batch] for n in ("q", "k", "v"))
    qf, kf, vf, kb, vb = f32(q), f32(k), (f32(v) if value_norm else None), raw(k), raw(v)
    share, gate = tables["head_share"], tables["t_gate"]
    t0 = time.perf_counter()
    out = oracle.retention_layer(
        qf, kf, vb, v=vf, W=w.window, mode=w.pool, kernel=w.pool_kernel, B=w.budget, cap=w.cap,
        w_head_row=f32(tables["w_head"][0]), share_row=None if share is None else f32(share[0]),
        gate_layer=None if gate is None else f32(gate[0]),
        risk_bins=None if gate is None else tables["risk_bins"].cpu().tolist()[:n_batch],
        value_norm=value_norm, k_bits=kb)
    dt = time.perf_counter() - t0
    sub = w.scaled(batch=n_batch)
    nbytes = algorithmic_bytes(sub, int(out["count"].sum()), value_norm)
    res = {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
           "sample": f"layer 0, batch elements 0..{n_batch - 1} of {w.batch} (all {w.n_kv_heads} KV heads), "
                     f"whole chain, {dt:.2f} s",
           "ms_per_layer_scaled": dt * 1e3 * w.batch / n_batch, "host": host_cpu()}
    if single_thread:   # the small configurations: the same chain on one core
        import subprocess
        code = ("import sys, time, numpy as np; sys.path.insert(0, %r); import oracle; d = np.load(sys.argv[1]);"
                "t0 = time.perf_counter();"
                "oracle.window_scores(d['q'], d['k']); print(time.perf_counter() - t0)" % ROOT)
        import tempfile
        import numpy as np
        with tempfile.NamedTemporaryFile(suffix=".npz") as f:
            np.savez(f.name, q=qf, k=kf)
            r = subprocess.run([sys.executable, "-c", code, f.name], capture_output=True, text=True,
                               env=dict(os.environ, OMP_NUM_THREADS="1"))
        if r.returncode == 0:
            res["single_thread_scan_ms"] = float(r.stdout.strip().splitlines()[-1]) * 1e3
    return res


def layer_shared_bench(args, w, n_layers, torch, B, wl) -> int:
    """The paper-literal mode: phase A over all layers (scan with value norms, alpha accumulation, risk),
    phase B over all layers (shared utility, selection, shared gather). One step = both phases."""
    dev = "cuda"
    tables = wl.make_tables(w, dev)
    layers = [wl.make_layer(w, l % w.n_layers, dev) for l in range(n_layers)]
    q0, k0, v0 = layers[0]["q"], layers[0]["k"], layers[0]["v"]
    # group masses (sums over each KV head's query heads) are all that alpha needs
    flags = B.FLAG_VALUE_NORM | (B.FLAG_GROUP_MASS if w.dtype == "bf16" and w.window <= 32 and w.group <= 4 else 0)
    params = [B.params_for(q0, k0, v0, pool=w.pool, pool_kernel=w.pool_kernel, budget=w.budget, cap=w.cap,
                           layer=l % w.n_layers, n_layers=w.n_layers, flags=flags) for l in range(n_layers)]
    one = B.make_params(batch=w.batch, n_q_heads=1, n_kv_heads=1, head_dim=w.head_dim, seq_len=w.seq_len,
                        window=w.window, dtype=w.dtype, pool=wl.POOL_NONE, pool_kernel=1, budget=w.budget, cap=w.cap,
                        n_layers=w.n_layers)
    buf = B.LayerBuffers(params[0], dev)
    Bz, T, P = w.batch, w.seq_len, w.prefix
    alpha = torch.zeros(Bz, T, device=dev)
    rho = [torch.empty(Bz, w.n_kv_heads, T, device=dev) for _ in range(n_layers)]
    risk, b_ent = torch.empty(Bz, device=dev), torch.empty(Bz, dtype=torch.int32, device=dev)
    edges = torch.linspace(0.0, float(torch.log(torch.tensor(float(T)))), 19, device=dev)
    util, tau = torch.empty(Bz, P, device=dev), torch.empty(Bz, device=dev)
    budget = torch.full((Bz, 1), w.budget, dtype=torch.int32, device=dev)
    idx = torch.full((Bz, w.cap), -1, dtype=torch.int32, device=dev)
    cnt = torch.empty(Bz, dtype=torch.int32, device=dev)
    wgt = 1.0 / (n_layers * w.n_q_heads)

    def step():
        alpha.zero_()
        for l in range(n_layers):
            t = layers[l]
            B.ckv_window_scores(params[l], t["q"], t["k"], t["v"], None, buf.scores, rho[l], buf.workspace)
            B.ckv_alpha_accumulate(params[l], buf.scores, wgt, alpha)
        B.ckv_risk_struct(params[0], alpha, edges, risk, b_ent)
        for l in range(n_layers):
            t = layers[l]
            B.ckv_shared_utility(params[l], alpha, rho[l], tables["w_head"], None, 0, 0, None, util, tau)
            B.ckv_select_topk(one, util, budget, tau, idx, cnt)
            B.ckv_compact_kv_shared(params[l], t["k"], t["v"], idx, cnt, buf.k_out, buf.v_out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_layer = ms_per_step / n_layers
    kept = int(cnt.sum().item()) * w.n_kv_heads
    layer_bytes = algorithmic_bytes(w, kept, True)
    value = layer_bytes / (ms_per_layer * 1e-3) / 1e9
    out = {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) of prefill-end scan+select+gather; ms/layer beside it",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_layer": round(ms_per_layer, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "mode": "layer_shared (Alg. 1 as printed)", "layers_per_step": n_layers,
                   "batch": w.batch, "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "seq_len": w.seq_len, "window": w.window, "budget_per_layer": w.budget, "value_norm": True,
                   "group_mass": bool(flags & B.FLAG_GROUP_MASS),
                   "algorithmic_bytes_per_layer": layer_bytes, "kept_rows_last_layer": kept},
        "roofline": None,
    }
    print(json.dumps(out))
    return 0


def decode_bench(args, w, n_layers, torch, B, wl) -> int:
    """Decode-side consumer: a step = one decoding query per head attending over the compact cache of every
    layer. The same call over the full cache and the discarded-mass kernel are timed beside it."""
    dev = "cuda"
    tables = wl.make_tables(w, dev)
    e = 2 if w.dtype == "bf16" else 4
    caches, full = [], []
    for l in range(n_layers):
        t = wl.make_layer(w, l % w.n_layers, dev)
        p = B.params_for(t["q"], t["k"], t["v"], pool=w.pool, pool_kernel=w.pool_kernel, budget=w.budget, cap=w.cap,
                         layer=l % w.n_layers, n_layers=w.n_layers)
        buf = B.LayerBuffers(p, dev)
        B.retention_layer(p, t["q"], t["k"], t["v"], tables, buf, fused_utility=True)
        torch.cuda.synchronize()
        caches.append((p, buf.k_out, buf.v_out, buf.count, wl.make_decode_queries(w, l % w.n_layers, 1, dev)))
        if l < 4:
            full.append((t["k"], t["v"]))
        del buf.scores, t
    kept = sum(int(c[3].sum().item()) for c in caches) / n_layers
    out = torch.empty(w.batch, w.n_q_heads, 1, w.head_dim, device=dev)
    lse_c, lse_f = torch.empty(w.batch, w.n_q_heads, 1, device=dev), torch.empty(w.batch, w.n_q_heads, 1, device=dev)
    mass, eps = torch.empty(w.batch, w.n_q_heads, 1, device=dev), torch.empty(w.batch, w.n_q_heads, device=dev)
    p0 = caches[0][0]
    ws = torch.empty(max(B.ckv_decode_workspace_bytes(p0, 1, w.seq_len), B.ckv_decode_workspace_bytes(p0, 1, w.cap)),
                     dtype=torch.uint8, device=dev)

    def step():
        for p, kc, vc, cnt, qd in caches:
            B.ckv_decode_attention(p, qd, kc, vc, cnt, out, lse_c, ws)

    # A decoding step is tens of short launches: queued one by one the host's launch cost bounds it, so the
    # step is captured once into a HIP graph and replayed (no memset nodes: the calls only launch kernels).
    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    eager_out, eager_lse = out.clone(), lse_c.clone()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_eager = (time.perf_counter() - t0) * 1e3 / args.steps
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(max(args.warmup, 1)):
        graph.replay()
        torch.cuda.synchronize()
        if not (torch.equal(out, eager_out) and torch.equal(lse_c, eager_lse)):
            print("bench.py: graph replay differs from the eager result", file=sys.stderr)
            return 4
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    if not (torch.equal(out, eager_out) and torch.equal(lse_c, eager_lse)):
        print("bench.py: graph replay differs from the eager result", file=sys.stderr)
        return 4
    ms_per_layer = ms_per_step / n_layers
    q_out_bytes = w.batch * w.n_q_heads * w.head_dim * (e + 4)
    compact_bytes = 2 * kept * w.head_dim * e + q_out_bytes          # every retained K and V row once
    full_bytes = 2 * w.batch * w.n_kv_heads * w.seq_len * w.head_dim * e + q_out_bytes
    ev = lambda: torch.cuda.Event(enable_timing=True)
    pairs_f, pairs_m = [], []
    for i in range(max(8, 2 * args.steps)):
        k, v = full[i % len(full)]
        p, kc, vc, cnt, qd = caches[i % len(full)]
        a, b_, c = ev(), ev(), ev()
        a.record()
        B.ckv_decode_attention(p, qd, k, v, None, out, lse_f, ws)
        b_.record()
        B.ckv_discarded_mass(p, 1, lse_f, lse_c, mass, eps)
        c.record()
        pairs_f.append((a, b_))
        pairs_m.append((b_, c))
    torch.cuda.synchronize()
    ms_full = sorted(a.elapsed_time(b_) for a, b_ in pairs_f)[len(pairs_f) // 2]
    ms_mass = sorted(a.elapsed_time(b_) for a, b_ in pairs_m)[len(pairs_m) // 2]
    # discarded mass of the last layer timed, from its own two normalisers
    p, kc, vc, cnt, qd = caches[0]
    B.ckv_decode_attention(p, qd, kc, vc, cnt, out, lse_c, ws)
    B.ckv_decode_attention(p, qd, full[0][0], full[0][1], None, out, lse_f, ws)
    B.ckv_discarded_mass(p, 1, lse_f, lse_c, mass, eps)
    torch.cuda.synchronize()
    value = compact_bytes / (ms_per_layer * 1e-3) / 1e9
    full_gbs = full_bytes / (ms_full * 1e-3) / 1e9
    line = {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) of one decoding step's attention over the compact cache",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_layer": round(ms_per_layer, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "mode": "decode (consumer of the compact cache)", "layers_per_step": n_layers,
                   "batch": w.batch, "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "seq_len": w.seq_len, "budget_per_kv_head": w.budget, "kept_rows_per_layer": kept,
                   "algorithmic_bytes_per_layer": int(compact_bytes), "launch": "HIP graph replay",
                   "ms_per_step_eager_launches": round(ms_eager, 4)},
        "roofline": {"bound": "hbm", "kernel": "decode_partial_kernel (full cache)", "achieved": round(full_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(full_gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "ms_per_launch": round(ms_full, 4), "discarded_mass_ms": round(ms_mass, 4),
                     "compact_cache_frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4)},
        "discarded_mass": {"mean": round(float(mass.mean().item()), 6), "max": round(float(mass.max().item()), 6),
                           "mean_eps_tail": round(float(eps.mean().item()), 6), "layer": 0},
    }
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c3",
                    choices=["c1", "c2", "c3", "c4", "c5", "s16k_b256", "s32k_b512", "s64k_b1024", "s128k_b2048", "s32k_b128"],
                    help="c3 is the workload the metric is quoted on; s*: length scaling at a fixed retained ratio "
                         "and the 128-token budget (C3's attention shape, batch 4)")
    ap.add_argument("--layers", type=int, default=0, help="distinct layer buffers (0 = the config's depth)")
    ap.add_argument("--value-norm", action="store_true")
    ap.add_argument("--given-lse", action="store_true", help="caller-supplied LSE: single pass over K")
    ap.add_argument("--unfused", action="store_true",
                    help="ckv_window_scores + ckv_apply_tables instead of ckv_window_utility (materialises the "
                         "per-head window mass)")
    ap.add_argument("--mode", default="per_head", choices=["per_head", "layer_shared", "decode"],
                    help="per_head: the north-star path (default). layer_shared: the paper's Alg. 1 as printed, one "
                         "alpha per prompt and one index set per layer (reported with the same metric). decode: the "
                         "decode-side consumer, one decoding query per head over every layer's compact cache")
    ap.add_argument("--streams", type=int, default=2,
                    help="HIP streams the layers of a step are dealt to in turn (1: every layer behind the previous one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-modes", action="store_true", help="skip the given-LSE and value-norm measurements")
    ap.add_argument("--graph", action=argparse.BooleanOptionalAction, default=None,
                    help="also time the step replayed from a HIP graph (default: for layers under 64 MiB)")
    ap.add_argument("--cpu-batch", type=int, default=0, help="batch elements in the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a kernel of known traffic for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported "
              "(every (layer, batch, KV head) unit is independent, so the path would shard over heads or "
              "batch without any exchange).", file=sys.stderr)
        return 2

    import torch

    from paper_2602_08686_amd import binding as B
    from paper_2602_08686_amd import workloads as wl

    B.load()  # fails loudly if libckv.so has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = "cuda"
    w = ({c.name[:2]: c for c in wl.CONFIGS} | {c.name.split("_gqa")[0]: c for c in wl.SWEEP})[args.config]
    n_layers = args.layers or w.n_layers
    flags = B.FLAG_VALUE_NORM if args.value_norm else 0

    if args.mode == "layer_shared":
        return layer_shared_bench(args, w, n_layers, torch, B, wl)
    if args.mode == "decode":
        return decode_bench(args, w, n_layers, torch, B, wl)
    tables = wl.make_tables(w, dev)
    layers = [wl.make_layer(w, l % w.n_layers, dev) for l in range(n_layers)]
    q0, k0, v0 = layers[0]["q"], layers[0]["k"], layers[0]["v"]

    def make_params(fl):
        return [B.params_for(q0, k0, v0, pool=w.pool, pool_kernel=w.pool_kernel, budget=w.budget, cap=w.cap,
                             layer=l % w.n_layers, n_layers=w.n_layers, flags=fl) for l in range(n_layers)]

    params = make_params(flags)
    # every layer has its own outputs and scratch, like its own K and V
    bufs = [B.LayerBuffers(params[l], dev) for l in range(n_layers)]
    lse_all = None

    def computed_lse():
        nonlocal lse_all
        if lse_all is None:
            lse_all = [torch.empty(w.batch, w.n_q_heads, w.window, device=dev) for _ in range(n_layers)]
            for l in range(n_layers):
                B.ckv_window_lse(params[l], layers[l]["q"], layers[l]["k"], lse_all[l], bufs[l].workspace)
            torch.cuda.synchronize()
        return lse_all

    # Layers are independent of one another (each has its K, V, outputs and scratch), so a caller that compacts
    # a whole model at the end of prefill can queue them on more than one stream: the short, latency-bound
    # kernels of one layer (selection, fix-up, gather) and the ends of its scans then overlap the next layer's
    # scan. All streams have the default priority.
    side_streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else None

    def time_whole_pass(prm, lse, steps, warmup, fused=True, streams=None):
        """ms per step of the whole call sequence over all layers (wall clock around a synchronised region);
        layer l goes to streams[l % len(streams)], or all to the current stream."""
        def step():
            for l in range(n_layers):
                t = layers[l]
                st = None if streams is None else streams[l % len(streams)]
                B.retention_layer(prm[l], t["q"], t["k"], t["v"], tables, bufs[l], lse=None if lse is None else lse[l],
                                  stream=st, fused_utility=fused)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, step

    lse = computed_lse() if args.given_lse else None
    ms_per_step, step = time_whole_pass(params, lse, args.steps, args.warmup, fused=not args.unfused, streams=side_streams)
    ms_per_layer = ms_per_step / n_layers
    one_stream_ms = ms_per_step
    if side_streams is not None:  # the same steps on one stream: every kernel of a layer behind the previous layer's last
        one_stream_ms, step = time_whole_pass(params, lse, args.steps, 1, fused=not args.unfused)
    kept = int(bufs[-1].count.sum().item())
    layer_bytes = algorithmic_bytes(w, kept, args.value_norm)
    value = layer_bytes / (ms_per_layer * 1e-3) / 1e9

    # Short shapes are bound by the launches themselves (five per layer): the same step replayed from a HIP
    # graph (the calls only launch kernels), every replay checked against the eager result.
    graph_ms = None
    if args.graph or (args.graph is None and layer_bytes < (64 << 20)):
        ref = [(b_.idx.clone(), b_.count.clone(), b_.utility.clone()) for b_ in bufs]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        ok = True
        for _ in range(max(args.warmup, 2)):
            g.replay()
            torch.cuda.synchronize()
            ok = ok and all(torch.equal(b_.idx, r[0]) and torch.equal(b_.count, r[1]) and torch.equal(b_.utility, r[2])
                            for b_, r in zip(bufs, ref))
        if not ok:
            print("bench.py: graph replay differs from the eager result", file=sys.stderr)
            return 4
        t0 = time.perf_counter()
        for _ in range(args.steps * 10):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / (args.steps * 10) / n_layers

    # Per-kernel timing of the two scan passes with events on the launch stream (torch's current one).
    reps = max(2, min(args.steps, 5))
    ev = lambda: torch.cuda.Event(enable_timing=True)
    lse_buf = torch.empty(w.batch, w.n_q_heads, w.window, device=dev)
    pairs1, pairs2 = [], []
    for _ in range(reps):
        for l in range(n_layers):
            t, buf = layers[l], bufs[l]
            a, b_, c = ev(), ev(), ev()
            a.record()
            B.ckv_window_lse(params[l], t["q"], t["k"], lse_buf, buf.workspace)
            b_.record()
            if args.unfused:
                B.ckv_window_scores(params[l], t["q"], t["k"], t["v"] if args.value_norm else None, lse_buf, buf.scores,
                                    buf.vnorm_ratio, buf.workspace)
            else:  # second pass with pooling, weights and group maximum on chip, plus its edge fix-up kernel
                B.ckv_window_utility(params[l], t["q"], t["k"], t["v"] if args.value_norm else None, lse_buf,
                                     tables["w_head"], tables.get("head_share"), tables.get("t_gate"),
                                     tables.get("n_ent", 0), tables.get("n_ppl", 0), tables.get("risk_bins"),
                                     buf.scores, buf.vnorm_ratio, buf.utility, buf.budget, buf.tau, buf.workspace)
            c.record()
            pairs1.append((a, b_))
            pairs2.append((b_, c))
    # Spread of one layer's whole call sequence (events around each layer of two more steps).
    per_layer = []
    for _ in range(2):
        marks = [ev() for _ in range(n_layers + 1)]
        marks[0].record()
        for l in range(n_layers):
            t = layers[l]
            B.retention_layer(params[l], t["q"], t["k"], t["v"], tables, bufs[l], lse=None if lse is None else lse[l],
                              fused_utility=not args.unfused)
            marks[l + 1].record()
        torch.cuda.synchronize()
        per_layer += [marks[l].elapsed_time(marks[l + 1]) for l in range(n_layers)]
    per_layer.sort()
    pct = lambda f: round(per_layer[min(len(per_layer) - 1, int(f * len(per_layer)))], 4)
    layer_ms = {"p10": pct(0.10), "p50": pct(0.50), "p90": pct(0.90), "samples": len(per_layer)}
    pairs3, pairs4 = [], []
    for _ in range(reps):
        for l in range(n_layers):
            t, buf = layers[l], bufs[l]
            a, b_, c = ev(), ev(), ev()
            a.record()
            B.ckv_select_topk(params[l], buf.utility, buf.budget, buf.tau, buf.idx, buf.count, buf.workspace)
            b_.record()
            B.ckv_compact_kv(params[l], t["k"], t["v"], buf.idx, buf.count, buf.k_out, buf.v_out)
            c.record()
            pairs3.append((a, b_))
            pairs4.append((b_, c))
    torch.cuda.synchronize()
    ms_select = sum(a.elapsed_time(b_) for a, b_ in pairs3) / len(pairs3)
    ms_gather = sum(a.elapsed_time(b_) for a, b_ in pairs4) / len(pairs4)
    gather_bytes = 4 * kept * w.head_dim * (2 if w.dtype == "bf16" else 4)
    ms_pass1 = sum(a.elapsed_time(b_) for a, b_ in pairs1) / len(pairs1)
    ms_pass2 = sum(a.elapsed_time(b_) for a, b_ in pairs2) / len(pairs2)
    bf16 = w.dtype == "bf16"
    dominant, dom_ms = ((("rowstats_lds_kernel" if bf16 else "rowstats_kernel"), ms_pass1)
                        if ms_pass1 >= ms_pass2 and not args.given_lse
                        else (("colsum_lds_kernel" if bf16 else "colsum_kernel"), ms_pass2))
    pass2_has_v = args.value_norm  # the second call also reads V for the value norms
    scan_ms = {"rowstats+lse": round(ms_pass1, 4),
               ("colsum" if args.unfused else "colsum+tables") + ("+vnorm" if pass2_has_v else ""): round(ms_pass2, 4)}
    dom_bytes = scan_bytes(w)
    if pass2_has_v and dominant.startswith("colsum"):
        dominant += " + vnorm_rows_kernel"   # timed together: K and V are each read once in that region
        dom_bytes += w.batch * w.n_kv_heads * w.seq_len * w.head_dim * (2 if bf16 else 4)
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    # which bound the scan sits under: the matrix-core rate needed to keep up with the HBM peak is
    # R = G * W flop per byte of K; the contraction is the bound where that exceeds what the kernels sustain
    mfma1 = scan_flops(w) / (ms_pass1 * 1e-3) / 1e12
    mfma2 = scan_flops(w) / (ms_pass2 * 1e-3) / 1e12
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": measured_traffic(dominant) if args.config == "c3" and not args.value_norm else None,
        "ms_per_launch": round(dom_ms, 4),
        "scan_ms": scan_ms,
        "select_ms": round(ms_select, 4), "gather_ms": round(ms_gather, 4),
        "gather_gbs": round(gather_bytes / (ms_gather * 1e-3) / 1e9, 1),
        "mfma_tflops": {"rowstats": round(mfma1, 1), "colsum": round(mfma2, 1),  # fused: its fix-up kernel included
                        "peak": MFMA_BF16_PEAK_TFLOPS,
                        "frac": round(max(mfma1, mfma2) / MFMA_BF16_PEAK_TFLOPS, 4) if bf16 else None},
        "whole_pass_frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "layer_ms": layer_ms,
    }
    if graph_ms is not None:
        roofline["graph_replay"] = {"ms_per_layer": round(graph_ms, 4),
                                    "gbs": round(layer_bytes / (graph_ms * 1e-3) / 1e9, 1),
                                    "frac_of_hbm_peak": round(layer_bytes / (graph_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # The other ways of calling the same path, measured in the same run with a few steps each: the caller
    # supplies LSE (one pass over K), and the value-norm factor of Eq. 4 switched on (V read once more).
    modes = None
    if not args.no_modes and not args.given_lse and not args.value_norm and not args.unfused:
        modes = {}
        m_steps = max(2, min(args.steps, 3))
        ms, _ = time_whole_pass(params, computed_lse(), m_steps, 1, streams=side_streams)
        gbs = layer_bytes / (ms / n_layers * 1e-3) / 1e9
        modes["given_lse"] = {"ms_per_layer": round(ms / n_layers, 4), "gbs": round(gbs, 1),
                              "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "steps": m_steps,
                              "algorithmic_bytes_per_layer": layer_bytes}
        vparams = make_params(flags | B.FLAG_VALUE_NORM)
        # one ratio buffer per stream (16 MiB that every layer on that stream overwrites)
        rho = [torch.empty(w.batch, w.n_kv_heads, w.seq_len, device=dev) for _ in range(max(args.streams, 1))]
        for l, b_ in enumerate(bufs):
            b_.vnorm_ratio = rho[l % len(rho)]
        need = B.ckv_workspace_bytes(vparams[0])
        if need > bufs[0].workspace.numel():
            for b_ in bufs:
                b_.workspace = torch.empty(need, dtype=torch.uint8, device=dev)
        ms, _ = time_whole_pass(vparams, None, m_steps, 1, streams=side_streams)
        vbytes = algorithmic_bytes(w, kept, True)
        gbs = vbytes / (ms / n_layers * 1e-3) / 1e9
        modes["value_norm"] = {"ms_per_layer": round(ms / n_layers, 4), "gbs": round(gbs, 1),
                               "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "steps": m_steps,
                               "algorithmic_bytes_per_layer": vbytes}

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) of prefill-end scan+select+gather; ms/layer beside it",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_layer": round(ms_per_layer, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers_per_step": n_layers, "batch": w.batch, "q_heads": w.n_q_heads,
                   "kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "seq_len": w.seq_len, "window": w.window,
                   "budget_per_kv_head": w.budget, "pool": ["none", "avg", "max"][w.pool] + str(w.pool_kernel),
                   "value_norm": bool(args.value_norm), "lse": "given" if args.given_lse else "computed",
                   "calls": ("window_scores+apply_tables" if args.unfused else "window_utility") + "+select_topk+compact_kv",
                   "buffers": "every layer its own K, V, outputs and scratch",
                   "streams": max(args.streams, 1),
                   "algorithmic_bytes_per_layer": layer_bytes, "kept_rows_last_layer": kept},
        "roofline": roofline,
        "one_stream": {"ms_per_layer": round(one_stream_ms / n_layers, 4),
                       "gbs": round(layer_bytes / (one_stream_ms / n_layers * 1e-3) / 1e9, 1)},
    }
    if modes is not None:
        out["modes"] = modes
    if not args.no_cpu_baseline:
        nb = args.cpu_batch or w.batch
        out["cpu_baseline"] = cpu_baseline(w, layers[0], tables, nb, args.value_norm,
                                           single_thread=args.config in ("c1", "c2"))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
