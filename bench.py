#!/usr/bin/env python3
"""Benchmark of the chunk-sparse expert FFN hot path on one MI355X.

A step is one pass of the whole path (router -> chunk union -> up projection -> down
projection, Sec. 3.3) over one batch of synthetic chunks that is already resident in HBM.
The default workload is the k = 8 speculative-verification configuration: d = 2048, 64 gated
experts of hidden size 128, bf16 weights, fp32 activations, 2048 chunks of 8 correlated
tokens.  Chunk c reads weight set c mod R of R distinct layers (R * 100.7 MB in HBM), so
that a chunk meets weights no other in-flight chunk has just pulled into the caches: the
weight stream comes from HBM, as it does when one sequence walks through a model's layers.

Prints ONE JSON line.  `value` is the active-expert weight bytes of the step divided by the
step's wall time (GB/s); the same line carries microseconds per chunk, tokens/s, the
fraction of the 8 TB/s HBM peak and of the read-stream ceiling measured in the same process
(a plain 128-bit-load read kernel over 8 GiB), the speedup over the dense FFN of equal size
(same kernels, all experts), the per-kernel split measured with HIP events on the launch
stream, the roofline of the dominant kernel, and the CPU oracle timed on a bounded sample.

`--all` also runs every measured configuration (single-token decode, k = 8, k = 32 trees, the
24-layer decode stack and the 512-token prefill), each with gated and with Eq. 2 experts, each
cold (chunks rotating through distinct weight sets) and warm (one weight set, cache assisted),
and appends one JSON record per run to a JSONL file (--all-out); the line printed at the end is
still the default one.
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

HBM_PEAK = 8.0e12  # bytes/s, MI355X HBM3E

# HBM bytes per launch of the up kernel from rocprofv3 (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the
# factors a plain 1 GiB device copy gives), keyed by (workload, replicas, gated), each with the
# profile summary it was read from: a number from an earlier build of the kernels, labelled as
# such in the output (`traffic_source`), never a measurement of the run that prints it.
MEASURED_TRAFFIC = {
    ("spec_k8", 128, True): (22088292 * 1024 * 2.0 + 171528 * 1024 * 1.0, "profiles/spec_k8_stream_kernels.md"),
}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--workload", default="spec_k8")
    p.add_argument("--replicas", type=int, default=0,
                   help="distinct weight sets the chunks rotate through (0: 128, or more where 128 sets stay "
                        "below 6 GiB: more sets than chunks are in flight at any moment)")
    p.add_argument("--chunks", type=int, default=0, help="override the number of chunks")
    p.add_argument("--swish", action="store_true", help="non-gated experts (Eq. 2) instead of the gated ones")
    p.add_argument("--sequential", action="store_true",
                   help="enqueue the chunks one after the other (one chunk per launch), as a layer stack does: "
                        "with --workload stack_decode_k8 --chunks 24 --replicas 24 a step is a 24-layer decode step")
    p.add_argument("--fused", action="store_true",
                   help="with --sequential: one blockffn_forward_chunks call per layer instead of the three calls "
                        "(three launches per layer instead of six)")
    p.add_argument("--graph", action="store_true",
                   help="with --sequential: capture the step's launches once as a HIP graph (kernel nodes only) and "
                        "replay it per step")
    p.add_argument("--dense-steps", type=int, default=3)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--extras", action="store_true",
                   help="also time the sparsity statistics (CLS_L sweep, reuse ratio), the training-objective forward "
                        "values and the expert-cache simulation on this workload's router outputs")
    p.add_argument("--cpu-sample-chunks", type=int, default=512)
    p.add_argument("--calibrate-copy", action="store_true",
                   help="only run a plain device copy of 1 GiB five times (reference for the rocprofv3 byte counters)")
    p.add_argument("--traffic-bytes", type=float, default=None,
                   help="HBM bytes per launch of the dominant kernel from rocprofv3 counters, if known")
    p.add_argument("--all", action="store_true",
                   help="also run every configuration (gated and Eq. 2 experts, cold and warm) and append one "
                        "JSON record each to the file --all-out names")
    p.add_argument("--all-out", default=os.path.join("gpurun_out", "bench_all.jsonl"),
                   help="JSONL file the records of --all are appended to (relative to this script)")
    p.add_argument("--no-ceiling", action="store_true", help="skip the read-stream ceiling measurement")
    p.add_argument("--ceiling-gib", type=int, default=8, help="size of the buffer the read-stream ceiling is measured on")
    return p.parse_args()


_CEILING = None


def stream_ceiling(gib):
    """GB/s of a plain 128-bit-load read stream over `gib` GiB on this device, best of the launch
    shapes the library offers, each the mean of 5 launches after one warm-up.  Measured once per process."""
    global _CEILING
    if _CEILING is not None:
        return _CEILING
    import torch

    from paper_2507_08771_amd import binding as B

    buf = torch.empty((gib << 30,), dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    sink = torch.zeros((1,), dtype=torch.int32, device="cuda")
    best, best_plain, per_variant = 0.0, 0.0, {}
    for variant in range(8):      # 0-3: plain loads, 4-7: non-temporal loads (what the weight streams use)
        us = timed_us(lambda: B.blockffn_stream_read(buf, variant, sink), reps=5)
        per_variant[str(variant)] = buf.numel() / us / 1e3
        best = max(best, per_variant[str(variant)])
        if variant < 4:
            best_plain = best
    del buf
    torch.cuda.empty_cache()
    _CEILING = {"GBps": best, "plain_loads_GBps": best_plain, "bytes": gib << 30, "by_launch_shape": per_variant}
    return _CEILING


def timed_us(fn, reps=5):
    import torch

    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e3


def extras(w, L, x, buf, chunk_layer):
    """Statistics and objectives on the router outputs of the timed workload.  The token stream is
    read as sequences of k tokens (the chunks: tokens that share a centre), and the CLS_L sweep
    also as one long sequence."""
    import torch

    from paper_2507_08771_amd import binding as B

    dev = x.device
    C, k, E, n_tok = w.n_chunks, w.k, w.E, w.n_tok
    l_max = 32
    inactive = torch.empty((2, l_max), dtype=torch.int64, device=dev)
    windows = torch.empty_like(inactive)
    cls = torch.empty((2, l_max), dtype=torch.float64, device=dev)
    num = torch.empty((E + 1,), dtype=torch.int64, device=dev)
    cnt = torch.empty_like(num)
    ratio = torch.empty((1,), dtype=torch.float64, device=dev)
    pre = torch.empty((n_tok, E), dtype=torch.float32, device=dev)
    losses = torch.empty((2,), dtype=torch.float64, device=dev)
    ws = torch.empty(B.blockffn_losses_workspace_bytes(), dtype=torch.uint8, device=dev)
    out = {}
    out["cls_sweep_us"] = timed_us(lambda: B.blockffn_cls_sweep(buf.token_mask, n_tok, n_tok, E, l_max, inactive,
                                                                windows, cls))
    out["cls_sliding_one_stream"] = {str(Lw): float(cls[1, Lw - 1]) for Lw in (1, 2, 4, 8, 16, 32)}
    B.blockffn_cls_sweep(buf.token_mask, n_tok, k, E, min(k, l_max), inactive, windows, cls)
    torch.cuda.synchronize()
    out["cls_disjoint_within_chunks"] = {str(Lw): float(cls[0, Lw - 1]) for Lw in (1, 2, 4, 8, 16, 32) if Lw <= k}
    out["reuse_ratio_us"] = timed_us(lambda: B.blockffn_reuse_ratio(buf.token_mask, n_tok, k, E, num, cnt, ratio))
    out["reuse_ratio_within_chunks"] = float(ratio.item())
    out["router_preact_us"] = timed_us(lambda: B.blockffn_router_preact(L, x, C, k, buf.scores, buf.token_mask, pre,
                                                                        chunk_layer))
    alpha = 16.0
    out["losses_us"] = timed_us(lambda: B.blockffn_router_losses(pre, n_tok, k, E, k, alpha, losses, ws))
    out["L_al(alpha=%g)" % alpha], out["L_cs(L=%d)" % k] = float(losses[0]), float(losses[1])
    # offloading: the chunks that read weight set 0, in order, are one layer's stream of unions
    sel = (chunk_layer == 0).nonzero().flatten() if chunk_layer is not None else torch.arange(C, device=dev)
    idx = buf.active_idx[sel].cpu().contiguous()
    n_act = buf.n_active[sel].cpu().contiguous()
    totals = torch.zeros(3, dtype=torch.int64)
    sim = {}
    for cap in (E // 4, E // 2, (3 * E) // 4, E):
        t0 = time.perf_counter()
        B.blockffn_offload_sim(idx, n_act, E, cap, None, totals)
        sim[str(cap)] = {"loads_per_chunk": float(totals[1]) / max(1, n_act.numel()),
                         "MB_per_chunk": float(totals[1]) * w.expert_bytes / max(1, n_act.numel()) / 1e6,
                         "hit_rate": 1.0 - float(totals[1]) / max(1, int(totals[0])),
                         "host_us": (time.perf_counter() - t0) * 1e6}
    out["offload_lru_by_capacity"] = sim
    return out


def cpu_baseline(w, layers, x, chunk_layer, n_sample, expert_bytes):
    """The oracle as it stands, timed on the host cores over a bounded sample of the same workload.
    Same source as the checker; built -O3 -march=native for the host it runs on (OpenMP over chunks)."""
    import numpy as np

    import oracle
    from paper_2507_08771_amd import workloads as wl

    oracle.use_native_build()
    cl = chunk_layer.cpu().numpy()
    order = np.argsort(cl, kind="stable")[:n_sample]          # chunks of the lowest-numbered weight sets
    groups = {}
    for c in order:
        groups.setdefault(int(cl[c]), []).append(int(c))
    xs = x.view(w.n_chunks, w.k, w.d)
    work = []
    for l, cs in groups.items():
        g = lambda n: None if layers.get(n) is None else wl.to_numpy(layers[n][l])
        L = oracle.Layer(g("w_router"), g("w_up"), g("w_down"), w_gate=g("w_gate"), b_router=g("b_router"))
        work.append((L, wl.to_numpy(xs[cs].reshape(-1, w.d))))
    active = 0
    t0 = time.perf_counter()
    for L, xc in work:
        r = oracle.forward(L, xc, w.k)
        active += int(r["n_active"].sum())
    dt = time.perf_counter() - t0
    n = len(order)
    # the oracle's dense pass (every expert evaluated) on a quarter of the sample: the CPU's own
    # sparse / dense ratio, to set beside the GPU's
    n_dense, dt_dense, left = 0, 0.0, max(1, n // 4)
    for L, xc in work:
        if left <= 0:
            break
        take = min(left, xc.shape[0] // w.k)
        xd = xc[:take * w.k]
        sc, _ = oracle.router(L, xd)
        t0 = time.perf_counter()
        oracle.dense_ffn(L, xd, sc)
        dt_dense += time.perf_counter() - t0
        n_dense += take
        left -= take
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": active * expert_bytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": "%d of %d chunks (router + union + chunk-sparse FFN in fp64, gcc -O3 -march=native -fopenmp), "
                      "%.1f s; dense FFN on %d of them, %.1f s" % (n, w.n_chunks, dt, n_dense, dt_dense),
            "us_per_chunk": dt / n * 1e6, "dense_us_per_chunk": dt_dense / n_dense * 1e6,
            "speedup_vs_dense": (dt_dense / n_dense) / (dt / n)}


def library_dense(w, layers, x, scores, y_ours, R, steps):
    """An independently written dense comparator: the dense FFN of equal parameter count (every
    expert, Eq. 1) through the vendor's GEMM library (torch.bmm on bf16, fp32 accumulation), the way
    a dense model would run it.  One batched call takes one chunk of every weight set (batch index =
    weight set), so every weight is read once per chunk, cold, exactly as in the library's own
    dense path; W_down is laid out [d][E * d_e] for it beforehand, outside the timed region.
    Activations are bf16 here (x rounded once): a timing comparator, checked loosely against
    blockffn_dense_ffn."""
    import torch
    import torch.nn.functional as F

    C, k, d, E, d_e = w.n_chunks, w.k, w.d, w.E, w.d_e
    N, m = E * d_e, C // R
    xb = x.view(m, R, k, d).to(torch.bfloat16)
    sc = scores.view(m, R, k, E).to(torch.bfloat16)
    wu_t = layers["w_up"].view(R, N, d).transpose(1, 2)
    wg_t = layers["w_gate"].view(R, N, d).transpose(1, 2) if w.gated else None
    wd_t = layers["w_down"].permute(0, 2, 1, 3).reshape(R, d, N).contiguous().transpose(1, 2)   # [R][N][d] view
    y = torch.empty((m, R, k, d), dtype=torch.bfloat16, device=x.device)

    def step():
        for j in range(m):
            u = torch.bmm(xb[j], wu_t)
            h = F.silu(torch.bmm(xb[j], wg_t)) * u if w.gated else F.silu(u)
            h = (h.view(R, k, E, d_e) * sc[j].unsqueeze(-1)).view(R, k, N)
            torch.bmm(h, wd_t, out=y[j])

    us = timed_us(step, reps=steps)
    # chunk c = j * R + r is row (j, r): same order as x
    ours = y_ours.view(m, R, k, d)
    diff = (y.float() - ours).pow(2).sum().sqrt() / ours.pow(2).sum().sqrt()
    return {"ms": us / 1e3, "rel_l2_diff_to_dense_ffn": float(diff),
            "what": "torch.bmm (vendor GEMM library), bf16 activations, one chunk per weight set per batched call"}


def default_replicas(w):
    """Weight sets the chunks rotate through when --replicas is not given: at least 128, and at
    least 6 GiB of weights.  The persistent workgroups of the up kernel hold about 50 chunks in
    flight at k = 8 (160 at k = 1).  With plain weight loads, fewer sets than that meant that two
    chunks in flight read the same set and the second found it in the caches (32 sets gave more
    than a plain read stream reaches on the same box; flat from 64 sets on).  The weight streams
    are non-temporal loads now and the k = 8 figure is flat from 16 to 256 sets; the default is
    kept."""
    set_bytes = w.E * w.expert_bytes
    return max(1, min(max(128, -(-(6 << 30) // set_bytes)), w.n_chunks))


def run(args, name, gated=None, replicas=0, sequential=False, chunks=0, steps=None, dense_steps=None, warm=False,
        with_cpu=False, with_extras=False, graph=False, fused=False):
    """One workload: generates it, times `steps` steps, returns the record."""
    import numpy as np
    import torch

    from paper_2507_08771_amd import binding as B
    from paper_2507_08771_amd import workloads as wl

    dev = "cuda"
    steps = args.steps if steps is None else steps
    dense_steps = args.dense_steps if dense_steps is None else dense_steps
    w = wl.WORKLOADS[name]
    if chunks:
        w = w.replace(n_chunks=chunks)
    if gated is not None:
        w = w.replace(gated=gated)
    R = 1 if warm else (replicas if replicas > 0 else default_replicas(w))
    R = max(1, min(R, w.n_chunks))

    layers = wl.make_layers(w, R, device=dev)
    chunk_layer = wl.make_chunk_layer(w, R, device=dev)
    x = wl.make_tokens(w, layers, chunk_layer, device=dev)
    L = B.Layer.from_dict(layers, gain=False)
    buf = B.Buffers(L, w.n_chunks, w.k)
    y_dense = torch.empty_like(buf.y)
    C, k = w.n_chunks, w.k
    stages = ("router", "union", "up", "down")

    # sequential mode: the way a model calls the library, one layer descriptor per layer (views
    # of the stacked weights) and no per-chunk layer table for the kernels to look up
    layer_of = chunk_layer.cpu().tolist()
    views = ([B.Layer.from_dict({n: (None if t is None else t[r:r + 1]) for n, t in layers.items()}, gain=False)
              for r in range(R)] if sequential else None)

    def step_sequential():
        for c in range(C):
            t0_, t1_ = c * k, (c + 1) * k
            Lc = views[layer_of[c]]
            if fused:
                B.blockffn_forward_chunks(Lc, x[t0_:t1_], 1, k, buf.scores[t0_:t1_], buf.token_mask[t0_:t1_],
                                          buf.union_mask[c:c + 1], buf.active_idx[c:c + 1], buf.n_active[c:c + 1],
                                          buf.stats, buf.y[t0_:t1_], buf.workspace)
                continue
            B.blockffn_router(Lc, x[t0_:t1_], 1, k, buf.scores[t0_:t1_], buf.token_mask[t0_:t1_])
            B.blockffn_chunk_union(buf.token_mask[t0_:t1_], 1, k, L.E, buf.union_mask[c:c + 1], buf.active_idx[c:c + 1],
                                   buf.n_active[c:c + 1], buf.stats)
            B.blockffn_sparse_ffn(Lc, x[t0_:t1_], buf.scores[t0_:t1_], buf.token_mask[t0_:t1_], buf.active_idx[c:c + 1],
                                  buf.n_active[c:c + 1], 1, k, buf.y[t0_:t1_], buf.workspace)

    use_graph, graph = graph, None
    if sequential and use_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step_sequential()                      # everything the calls set up lazily happens before capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step_sequential()

    def step(ev=None):
        if sequential:
            if ev: ev[0].record()
            if graph is not None: graph.replay()
            else: step_sequential()
            if ev:
                for e in ev[1:]: e.record()
            return
        if ev: ev[0].record()
        B.blockffn_router(L, x, C, k, buf.scores, buf.token_mask, chunk_layer)
        if ev: ev[1].record()
        B.blockffn_chunk_union(buf.token_mask, C, k, L.E, buf.union_mask, buf.active_idx, buf.n_active, buf.stats)
        if ev: ev[2].record()
        B.blockffn_sparse_ffn_up(L, x, buf.scores, buf.token_mask, buf.active_idx, buf.n_active, C, k,
                                 buf.workspace, chunk_layer)
        if ev: ev[3].record()
        B.blockffn_sparse_ffn_down(L, buf.active_idx, buf.n_active, C, k, buf.y, buf.workspace, chunk_layer)
        if ev: ev[4].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    buf.stats.zero_()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall / steps * 1e3
    step_ms = sorted(ev[0].elapsed_time(ev[4]) for ev in events)     # HIP events around each step
    stage_us = {s: sum(ev[i].elapsed_time(ev[i + 1]) for ev in events) / steps * 1e3 for i, s in enumerate(stages)}
    up_us = sorted(ev[2].elapsed_time(ev[3]) * 1e3 for ev in events)
    n_active_sum = int(buf.n_active.sum().item())
    stats = buf.stats.cpu().numpy()
    tls = float(stats[0]) / (steps * w.n_tok * w.E)
    cls = float(stats[1]) / (steps * C * w.E)
    sw = 2 if w.wdtype == "bf16" else 4
    active_bytes = n_active_sum * w.expert_bytes
    up_bytes = n_active_sum * (w.n_mats - 1) * w.d * w.d_e * sw

    # dense FFN of equal parameter count: same kernels, every expert, no masks
    dense_ms = None

    def dense_step():
        if not sequential:
            B.blockffn_dense_ffn(L, x, buf.scores, C, k, y_dense, buf.workspace, chunk_layer)
            return
        for c in range(C):   # the dense layer stack: router, then every expert of the layer
            t0_, t1_ = c * k, (c + 1) * k
            Lc = views[layer_of[c]]
            B.blockffn_router(Lc, x[t0_:t1_], 1, k, buf.scores[t0_:t1_], buf.token_mask[t0_:t1_])
            B.blockffn_dense_ffn(Lc, x[t0_:t1_], buf.scores[t0_:t1_], 1, k, y_dense[t0_:t1_], buf.workspace)

    if dense_steps > 0:
        dense_step()
        torch.cuda.synchronize()
        if graph is not None:      # the dense stack replayed as a graph as well
            dense_graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(dense_graph):
                dense_step()
            dense_step = dense_graph.replay
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(dense_steps):
            dense_step()
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / dense_steps
    library = None
    if dense_steps > 0 and not sequential and w.wdtype == "bf16" and C % R == 0 and w.k <= 32 and R >= 32:   # cold only
        library = library_dense(w, layers, x, buf.scores, y_dense, R, dense_steps)
    ffn_ms = (stage_us["up"] + stage_us["down"]) / 1e3
    if sequential:   # whole steps on both sides (router included): there is no per-kernel split here
        ffn_ms = ms_per_step

    up_s = stage_us["up"] * 1e-6
    if sequential:   # no per-kernel split in this mode: price the whole step against all active bytes
        up_s, up_bytes = ms_per_step * 1e-3, active_bytes
    traffic, traffic_source = None, None
    if args.traffic_bytes is not None:
        traffic, traffic_source = args.traffic_bytes, "--traffic-bytes"
    elif not chunks and (w.name, R, w.gated) in MEASURED_TRAFFIC:
        traffic, traffic_source = MEASURED_TRAFFIC[(w.name, R, w.gated)]
        traffic_source += " (rocprofv3 counters of an earlier run of this workload, not of this run)"
    value = active_bytes / (ms_per_step * 1e-3) / 1e9
    dense_bytes = C * w.E * w.expert_bytes
    out = {
        "metric": "µs/chunk + active-weight HBM GB/s (%% peak) at k=%d; speedup vs dense FFN" % k,
        "value": value,
        "unit": "GB/s (active-expert weight bytes / step wall time)",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "step_ms_hip_events": {"median": step_ms[len(step_ms) // 2], "min": step_ms[0], "max": step_ms[-1]},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights, f32 activations and accumulation" if w.wdtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: d=%d E=%d d_e=%d %s experts, k=%d x %d chunks, sigma=%.2f, %d weight sets (%.2f GB)%s%s"
                               % (w.name, w.d, w.E, w.d_e, "gated" if w.gated else "swish", k, C, w.sigma, R,
                                  R * w.E * w.expert_bytes / 1e9,
                                  (", chunks enqueued one after the other" + (", one fused call per layer" if fused else "")
                                   + (" (replayed as a HIP graph)" if graph is not None else ""))
                                  if sequential else "",
                                  ", WARM: one weight set for every chunk, served largely by the caches (not an HBM figure)"
                                  if warm and C > 1 else ""),
                   "name": w.name, "expert_kind": "gated" if w.gated else "swish",
                   "replicas": R, "sequential": sequential, "graph": graph is not None, "fused": bool(fused and sequential),
                   "mode": "warm" if warm and C > 1 else "cold"},
        "us_per_chunk": ms_per_step * 1e3 / C,
        "tokens_per_s": w.n_tok / (ms_per_step * 1e-3),
        "pct_hbm_peak": 100.0 * active_bytes / (ms_per_step * 1e-3) / HBM_PEAK,
        "stage_us": stage_us,
        "mean_active_experts": n_active_sum / C, "tls": tls, "cls_k": cls,
        "dense_ffn_ms": dense_ms, "sparse_ffn_ms": ffn_ms,
        "dense_ffn_GBps": None if dense_ms is None else dense_bytes / (dense_ms * 1e-3) / 1e9,
        "speedup_vs_dense": None if dense_ms is None else dense_ms / ffn_ms,
        "dense_library_gemm": None if library is None else dict(
            library, speedup_of_sparse=library["ms"] / ffn_ms,
            GBps=dense_bytes / (library["ms"] * 1e-3) / 1e9),
        "E_over_mean_active": w.E * C / max(n_active_sum, 1),
        "paper_context": "up to 3.67x end-to-end over dense decoding on Jetson Orin NX (another machine, Table 6)",
        "roofline": {"kernel": "up projection over the union (W_up%s rows of the active experts)"
                               % (" and W_gate" if w.gated else ""),
                     "bound": "hbm", "achieved": up_bytes / up_s / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                     "frac": up_bytes / up_s / HBM_PEAK,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": up_bytes,
                     "avg_launch_us": stage_us["up"],
                     "launch_us_hip_events": {"median": up_us[len(up_us) // 2], "min": up_us[0]}},
    }
    if not args.no_ceiling:
        del y_dense
        ceil = stream_ceiling(args.ceiling_gib)
        out["stream_ceiling_GBps"] = ceil["GBps"]
        out["stream_ceiling"] = ceil
        out["frac_of_ceiling"] = value / ceil["GBps"]
        out["roofline"]["frac_of_stream_ceiling"] = out["roofline"]["achieved"] / ceil["GBps"]
    if with_extras:
        out["extras"] = extras(w, L, x, buf, chunk_layer)
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(w, layers, x, chunk_layer, min(args.cpu_sample_chunks, C), w.expert_bytes)
    return out


# (workload, keyword arguments of run()) of --all: the measured configurations, cold
ALL_RUNS = [
    ("decode_k1", dict()),
    ("spec_k8", dict()),
    ("tree_k32", dict(steps=5, dense_steps=2)),
    ("stack_decode_k8", dict(chunks=24, replicas=24, sequential=True)),
    ("stack_decode_k8", dict(chunks=24, replicas=24, sequential=True, graph=True)),
    ("stack_decode_k8", dict(chunks=24, replicas=24, sequential=True, graph=True, fused=True)),
    ("stack_prefill_512", dict(chunks=8, replicas=8, steps=10, dense_steps=2)),
    ("paper_ar_k1", dict()),
    ("paper_tree_k32", dict(steps=10, dense_steps=2)),
]


def run_all(args):
    import torch

    path = os.path.join(ROOT, args.all_out)
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "a") as f:
        for name, kw in ALL_RUNS:
            kinds = (None,) if name.startswith("paper_") else (True, False)   # the paper shapes are Eq. 2 only
            for gated in kinds:
                for warm in (False, True):
                    if warm and kw.get("sequential"):
                        continue    # a layer stack has one weight set per layer by definition
                    rec = run(args, name, gated=gated, warm=warm, **kw)
                    f.write(json.dumps(rec) + "\n")
                    f.flush()
                    lib = rec.get("dense_library_gemm")
                    print("%-18s %-6s %-4s %8.1f GB/s  %5.1f %% of 8 TB/s  %8.2f us/chunk  speedup %s (bound %.2f)  "
                          "vs library GEMM dense %s"
                          % (name, rec["config"]["expert_kind"], rec["config"]["mode"], rec["value"], rec["pct_hbm_peak"],
                             rec["us_per_chunk"],
                             "-" if rec["speedup_vs_dense"] is None else "%.2f" % rec["speedup_vs_dense"],
                             rec["E_over_mean_active"],
                             "-" if not lib else "%.2f (%.0f GB/s)" % (lib["speedup_of_sparse"], lib["GBps"])),
                          file=sys.stderr, flush=True)
                    torch.cuda.empty_cache()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (chunks are independent and would "
              "shard data-parallel with replicated weights); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones((1 << 28,), dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4}))
        return
    if args.all:
        run_all(args)
    out = run(args, args.workload, gated=False if args.swish else None, replicas=args.replicas,
              sequential=args.sequential, chunks=args.chunks, with_cpu=not args.no_cpu_baseline,
              with_extras=args.extras, graph=args.graph, fused=args.fused)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
