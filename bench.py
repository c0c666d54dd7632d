#!/usr/bin/env python3
"""Benchmark of the learned-cache lookup hot path on one MI355X.

A step is one pass of a whole cache stack over one batch of synthetic activations
already resident in HBM: for every layer, pool -> predictor FCs -> softmax/argmax ->
selector -> hit flags -> miss compaction, the next layer looking up only the misses,
with the miss counts chained on the device (no host round trip inside a step).

Prints ONE JSON line: lookups/s for the whole job, the pooling kernel's achieved HBM
bandwidth against the MI355X peak (measured with HIP events around every pooling
launch), and the CPU oracle timed on the host cores on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth, GB/s
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X published dense matrix peaks

# HBM traffic per launch of a pooling kernel instance, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this file (not re-measured by a plain run: counters need the profiler).  Keyed by
# (workload, kernel instance); each entry names the summary under profiles/ it was read from.  The
# figure is attached only when that instance is the dominant one of the run.
PROFILED_TRAFFIC = {
    ("resnet50", "ncs_wave[C=256,S=3136,bf16]"): (819_310_000, "profiles/pool_ncs_wave_bf16_resnet50_hbm_traffic.md"),
    ("bert_base", "nsc_unit[C=768,S=128,bf16]"): (142_730_000, "profiles/pool_nsc_unit_bf16_bert_base_hbm_traffic.md"),
    ("resnet50_conv", "conv_rows[C=256,S=3136,bf16]"): (833_320_000, "profiles/conv_rows_bf16_resnet50_conv_hbm_traffic.md"),
    ("resnet50_pool", "ncs_adaptive[C=256,S=3136,bf16]"): (825_590_000, "profiles/pool_ncs_adaptive_bf16_resnet50_pool_hbm_traffic.md"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_workload(name, torch, g, W):
    """Caches, device buffers and activations of one workload.  For "gather" storage every
    layer holds the full batch; for "dense" storage a first untimed pass generates each layer
    only for the rows still active and stores them in miss-list order."""
    spec = W.get_workload(name)
    K = spec.layers[0].K
    labels = W.zipf_labels(spec.batch, K, spec.zipf_s, spec.seed)
    weights = [W.cache_weights(spec, l) for l in range(len(spec.layers))]
    caches = [g.Cache.from_layer(L, w, spec.batch) for L, w in zip(spec.layers, weights)]
    stack = g.CacheStack(caches, spec.batch, storage=spec.storage)
    acts = []
    if spec.storage == "gather":
        req = np.arange(spec.batch)
        for l in range(len(spec.layers)):
            acts.append(W.activation_bulk(spec, l, labels, req, device="cuda"))
    else:
        # pass 1 (untimed): layer by layer, reading the miss list back to generate the next layer
        es = stack.counts.element_size()
        base = stack.counts.data_ptr()
        active = np.arange(spec.batch)
        for l, cache in enumerate(caches):
            a = W.activation_bulk(spec, l, labels, active if len(active) else np.arange(1), device="cuda")
            acts.append(a)
            cache.lookup(a, None, spec.batch, base + l * es, stack.pred_class[l], stack.confidence[l], stack.hit[l])
            cache.compact(stack.hit[l], stack.ids[l], spec.batch, base + l * es, stack.ids[l + 1], base + (l + 1) * es)
            torch.cuda.synchronize()
            n_next = int(stack.counts[l + 1].item())
            active = stack.ids[l + 1][:n_next].cpu().numpy().astype(np.int64)
    torch.cuda.synchronize()
    return spec, labels, weights, caches, stack, acts


def time_stack(stack, acts, steps, warmup, torch):
    for _ in range(warmup):
        stack.run(acts)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        stack.run(acts)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def time_pool_launches(spec, caches, stack, acts, keys, reps, torch):
    """HIP events around the pooling launches, all layers in stack order so that no layer is
    re-read from cache; same kernels, launch shapes, row lists and device counts as in a stack
    pass.  Consecutive layers that run the same kernel instance share one event pair (their
    launches queue back to back, as they do behind the head kernels in a real pass), so the
    figure is kernel time plus launch-to-launch gaps, not host enqueue latency.
    Returns per-layer mean duration in ms (a group's time is split by algorithmic bytes)."""
    L = len(caches)
    pooled = [torch.empty(spec.batch, c.F, dtype=torch.float32, device="cuda") for c in caches]
    es, base = stack.counts.element_size(), stack.counts.data_ptr()
    groups = []                         # [first, last] layer index of each run of equal keys
    for l in range(L):
        if groups and keys[groups[-1][0]] == keys[l]:
            groups[-1][1] = l
        else:
            groups.append([l, l])
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in groups]
          for _ in range(reps)]
    # Launches of a few microseconds end before the host has enqueued the next one, and the idle time would
    # land between the events: give the host a head start of a few milliseconds of plain reads, so that every
    # timed launch and event is already queued when the GPU reaches it.
    import paper_2101_07344_amd as g
    blocker = torch.empty(64 << 20, dtype=torch.float32, device="cuda")
    sink = torch.zeros(256 * 32 * 1024, dtype=torch.float32, device="cuda")
    lead_ms = 0.012 * (reps + 1) * (L + 2 * len(groups))      # ~12 us of host time per call
    torch.cuda.synchronize()
    for _ in range(int(lead_ms / 0.04) + 1):                  # a 256 MB read takes ~40 us
        g.gati_probe_stream_read(blocker, blocker.numel() * 4, sink, 1)
    for r in range(-1, reps):           # r = -1: warm-up
        for gi, (lo, hi) in enumerate(groups):
            if r >= 0:
                ev[r][gi][0].record()
            for l in range(lo, hi + 1):
                row_index = stack.ids[l] if spec.storage == "gather" else None
                caches[l].pool(acts[l], row_index, spec.batch, base + l * es, pooled[l])
            if r >= 0:
                ev[r][gi][1].record()
    torch.cuda.synchronize()
    ms = np.array([[a.elapsed_time(b) for a, b in row] for row in ev]).mean(axis=0)
    return groups, ms


def time_graph(stack, acts, steps, warmup, torch):
    """The same pass captured once into a HIP graph and replayed."""
    stream = torch.cuda.current_stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        stack.run(acts)
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_uncompacted(spec, caches, acts, steps, warmup, torch):
    """The stack without layer-to-layer compaction: every layer looks up the whole batch, as a batch does
    that runs until its slowest member is done (Section 7, the paper's batch mode).  What the miss lists save."""
    n = spec.batch
    pc = torch.empty(n, dtype=torch.int32, device="cuda")
    conf = torch.empty(n, device="cuda")
    hit = torch.empty(n, dtype=torch.uint8, device="cuda")
    def one_pass():
        for cache, a in zip(caches, acts):
            cache.lookup(a, None, n, None, pc, conf, hit)
    for _ in range(warmup):
        one_pass()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        one_pass()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_overlap(stack, acts, steps, warmup, torch, gemm_dim=4096):
    """Lookups beside a stand-in for the base DNN (the paper's serving arrangement, Section 6:
    base model on one stream, cache lookups on a second one).  The stand-in is one bf16
    gemm_dim^3 library GEMM per layer; layer l's lookup may start when 'its' GEMM is done.
    Returns ms per pass for: the stand-in alone, everything on one stream, lookups on a side stream."""
    a = torch.randn(gemm_dim, gemm_dim, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(gemm_dim, gemm_dim, device="cuda", dtype=torch.bfloat16)
    out = torch.empty(gemm_dim, gemm_dim, device="cuda", dtype=torch.bfloat16)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    L = len(stack.caches)
    done = [torch.cuda.Event() for _ in range(L)]

    def base_only():
        for _ in range(L):
            torch.matmul(a, b, out=out)

    def sync_pass():
        for l in range(L):
            torch.matmul(a, b, out=out)
            stack.run_layer(l, acts[l], stream=main)

    def async_pass():
        for l in range(L):
            torch.matmul(a, b, out=out)
            done[l].record(main)
            side.wait_event(done[l])
            stack.run_layer(l, acts[l], stream=side)
        main.wait_stream(side)

    res = {}
    for name, fn in (("base_only_ms", base_only), ("same_stream_ms", sync_pass), ("side_stream_ms", async_pass)):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(e0.elapsed_time(e1) / steps, 4)
    res["standin"] = f"{L} x bf16 GEMM {gemm_dim}^3 (torch.matmul), one per layer"
    res["lookup_cost_same_stream_ms"] = round(res["same_stream_ms"] - res["base_only_ms"], 4)
    res["lookup_cost_side_stream_ms"] = round(res["side_stream_ms"] - res["base_only_ms"], 4)
    return res


def cpu_baseline(spec, weights, acts, stack, counts, budget_requests, torch, W):
    """The CPU oracle, one thread, on the first `budget_requests` requests of the same batch
    through the whole stack (its own hits and compaction).  TEST INFRASTRUCTURE timed as a
    reported baseline only."""
    import oracle
    from oracle import admit
    defs = admit.cache_defs(spec, mirror=True)
    m = min(budget_requests, spec.batch)
    host = []
    if spec.storage == "gather":
        for a in acts:
            host.append(W.to_host_array(a[:m]))
    else:
        # dense storage: row i of layer l belongs to request ids[l][i]; take the rows of requests < m
        for l, a in enumerate(acts):
            ids = stack.ids[l][:counts[l]].cpu().numpy()
            sel = np.nonzero(ids < m)[0]
            rows = a[torch.from_numpy(sel).cuda()] if len(sel) else a[:0]
            full = torch.zeros((m,) + tuple(a.shape[1:]), dtype=a.dtype)
            if len(sel):
                full[torch.from_numpy(ids[sel].astype(np.int64))] = rows.cpu()
            host.append(W.to_host_array(full))
    t0 = time.perf_counter()
    res = oracle.stack(defs, weights, host, m, storage="gather")
    dt = time.perf_counter() - t0
    lookups = int(sum(len(r.ids_in) for r in res))
    return {"value": lookups / dt, "unit": "lookups/s", "cores": 1, "kind": "oracle",
            "sample": f"first {m} of {spec.batch} requests through all {len(defs)} layers "
                      f"({lookups} lookups, {dt:.1f} s, single thread, gcc -O2, fp64 accumulation)"}


def cpu_baseline_all_cores(spec, weights, acts, budget_requests, torch, W):
    """The same oracle over the same requests, sharded by request over the host cores: each shard of
    requests goes through the whole stack on its own (requests are independent), one single-threaded
    oracle call chain per host thread (the C library runs outside the interpreter lock).  Gather
    storage only.  A pool sized to the machine's CPU share for one GPU, at most 16."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    from oracle import admit
    defs = admit.cache_defs(spec, mirror=True)
    m = min(budget_requests, spec.batch)
    threads = max(1, min(16, os.cpu_count() or 1, m))
    host = [W.to_host_array(a[:m]) for a in acts]
    bounds = np.linspace(0, m, threads + 1).astype(int)

    def shard(k):
        lo, hi = int(bounds[k]), int(bounds[k + 1])
        if hi <= lo:
            return 0
        res = oracle.stack(defs, weights, [h[lo:hi] for h in host], hi - lo, storage="gather")
        return int(sum(len(r.ids_in) for r in res))

    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        lookups = sum(ex.map(shard, range(threads)))
    dt = time.perf_counter() - t0
    return {"value": lookups / dt, "unit": "lookups/s", "cores": threads, "kind": "oracle x cores",
            "host_cpu_count": os.cpu_count(),
            "sample": f"first {m} of {spec.batch} requests through all {len(defs)} layers, request-sharded over "
                      f"{threads} host threads ({lookups} lookups, {dt:.2f} s)"}


def stream_read_ceiling(acts, torch, g, min_bytes=512 << 20, reps=10):
    """What a plain streaming read reaches on this machine, this run: the library's read-only probe kernel
    (non-temporal 16-byte loads, nothing written) over a tensor well beyond the last-level cache."""
    buf = acts[0] if acts[0].numel() * acts[0].element_size() >= min_bytes else torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    nbytes = buf.numel() * buf.element_size() // 16 * 16
    sink = torch.zeros(256 * 32 * 1024, dtype=torch.float32, device="cuda")
    best = None
    for bpc in (0, 1, 2, 4, 8, 16):     # which launch shape reads fastest differs from box to box (0: a wave per 8 KB chunk)
        for _ in range(2):
            assert g.gati_probe_stream_read(buf, nbytes, sink, bpc) == g.GATI_OK
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.gati_probe_stream_read(buf, nbytes, sink, bpc)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts.sort()
        t = ts[len(ts) // 2] * 1e-3
        if best is None or t < best[0]:
            best = (t, bpc)
    t, bpc = best
    return {"GBps": round(nbytes / t / 1e9, 1), "bytes": nbytes, "us": round(t * 1e6, 1),
            "kernel": f"gati_probe_stream_read, " + (f"{bpc} workgroups per CU" if bpc else "one wave per 8 KB chunk") + " (best of 6 launch shapes), "
                      f"median of {reps} launches"}


def dependent_launch_floor(torch, g, links=200, reps=5):
    """What a launch costs that waits for its predecessor's output and computes nothing: chains of the
    library's probe kernel (`gati_probe_launch_chain`), per link, at the grid sizes of the predictor /
    selector kernels and with 0, 1 and 2 dependent loads per lane.  The head of a layer is three such
    launches plus their arithmetic."""
    cell = torch.zeros(2, dtype=torch.int32, device="cuda")
    out = {}
    for wgs in (16, 128, 512):
        for loads in (0, 1, 2):
            assert g.gati_probe_launch_chain(cell, 20, wgs, loads) == g.GATI_OK
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                g.gati_probe_launch_chain(cell, links, wgs, loads)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3 / links)
            ts.sort()
            out[f"{wgs}wg_{loads}loads_us"] = round(ts[len(ts) // 2], 2)
    out["what"] = (f"median of {reps} chains of {links} launches of gati_probe_launch_chain, microseconds per launch; "
                   "workgroups of 256 lanes, every lane follows the given number of dependent 4-byte loads from a cell the previous launch wrote")
    return out


def plain_read_same_sizes(spec, acts, counts, torch, g, reps=5):
    """A plain read of as many bytes as each layer's pooling launch reads, launched back to back in
    layer order between one event pair (the way the pooling launches are timed): what a kernel that
    does nothing but read gets out of launches of these sizes, ramp and drain included."""
    sink = torch.zeros(256 * 32 * 1024, dtype=torch.float32, device="cuda")
    nbytes = [int(counts[l]) * L.row_bytes // 16 * 16 for l, L in enumerate(spec.layers)]
    total = sum(nbytes)
    if total == 0:
        return None
    best = None
    blocker = torch.empty(64 << 20, dtype=torch.float32, device="cuda")
    for bpc in (0, 1, 32):
        ts = []
        for r in range(-1, reps):
            # host head start, as in time_pool_launches
            for _ in range(int(0.012 * (len(acts) + 2) / 0.04) + 1):
                g.gati_probe_stream_read(blocker, blocker.numel() * 4, sink, 1)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for a, nb in zip(acts, nbytes):
                if nb:
                    g.gati_probe_stream_read(a, nb, sink, bpc)
            e1.record()
            torch.cuda.synchronize()
            if r >= 0:
                ts.append(e0.elapsed_time(e1))
        ts.sort()
        t = ts[len(ts) // 2] * 1e-3
        if best is None or t < best:
            best = t
    return round(total / best / 1e9, 1)


def pool_yardstick(spec, acts, torch):
    """The vendor reduction (torch mean over the pooled axis, fp32 result) on layer 0's full tensor."""
    L = spec.layers[0]
    x = acts[0]
    dim = 2 if L.layout == "ncs" else 1
    fn = lambda: x.mean(dim=dim, dtype=torch.float32)
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(10):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ts.sort()
    t = ts[len(ts) // 2] * 1e-3
    nbytes = x.numel() * x.element_size()
    return {"shape": list(x.shape), "library_us": round(t * 1e6, 1), "library_GBps": round(nbytes / t / 1e9, 1)}


def time_compaction(cache, stack, batch, torch, reps=20):
    """The stand-alone miss compaction over a full batch of layer 0's hit flags (in the stack it is
    fused into the finish kernel and costs no launch of its own)."""
    ids_out = torch.empty(batch, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(3):
        cache.compact(stack.hit[0], None, batch, None, ids_out, cnt)
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        cache.compact(stack.hit[0], None, batch, None, ids_out, cnt)
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ts.sort()
    return round(ts[len(ts) // 2] * 1e3, 2)


def run_workload(name, steps, warmup, with_cpu, cpu_requests, torch, g, W, copy_probe=False,
                 graph=False, overlap=False, yardstick=False, train=False, ceiling=False, uncompacted=False):
    t_build = time.perf_counter()
    spec, labels, weights, caches, stack, acts = build_workload(name, torch, g, W)
    if copy_probe:
        dst = torch.empty_like(acts[0])
        nbytes = acts[0].numel() * acts[0].element_size()
        assert g.gati_probe_copy(dst, acts[0], nbytes) == g.GATI_OK
        torch.cuda.synchronize()
        log(f"[{name}] copy probe (probe_copy_kernel): {nbytes} bytes read, same written")
        del dst
    log(f"[{name}] inputs ready in {time.perf_counter() - t_build:.1f}s "
        f"({sum(a.numel() * a.element_size() for a in acts) / 1e9:.2f} GB of activations)")
    if spec.layers[0].predictor == "fc_mlp":
        cpu_requests = min(cpu_requests, 4)         # the oracle needs ~1 G multiply-adds per row and layer
    ms_step, wall_ms = time_stack(stack, acts, steps, warmup, torch)
    counts = stack.counts.cpu().numpy().astype(np.int64)
    n_layers = len(caches)
    lookups = int(counts[:n_layers].sum())
    hits = [(int(counts[l] - counts[l + 1]) / int(counts[l])) if counts[l] else None for l in range(n_layers)]

    elem = spec.layers[0].elem_bytes
    keys = [f"{c.pool_variant}[C={L.C},S={L.S},{L.dtype}]" for L, c in zip(spec.layers, caches)]
    algo = [int(counts[l]) * L.C * L.S * elem + int(counts[l]) * L.F * 4      # activation read + pooled write
            + (L.H * L.C * L.S * elem if L.predictor == "fc_mlp" else 0)      # FC(h): W1 is streamed once too
            for l, L in enumerate(spec.layers)]
    flops = [2 * int(counts[l]) * L.C * L.S * L.H if L.predictor == "fc_mlp" else 0 for l, L in enumerate(spec.layers)]
    groups, group_ms = time_pool_launches(spec, caches, stack, acts, keys, max(3, min(steps, 20)), torch)
    per_layer, by_kernel = [], {}
    for (lo, hi), gms in zip(groups, group_ms):
        gbytes = sum(algo[lo:hi + 1])
        k = by_kernel.setdefault(keys[lo], {"bytes": 0, "flops": 0, "ms": 0.0, "launches": 0})
        for l in range(lo, hi + 1):
            n = int(counts[l])
            share = float(gms) * (algo[l] / gbytes) if gbytes else 0.0
            per_layer.append({"layer": l, "n": n, "kernel": keys[l], "pool_us": round(share * 1e3, 2),
                              "pool_GBps": round(algo[l] / (share * 1e-3) / 1e9, 1) if share else 0.0,
                              "hit_rate": None if hits[l] is None else round(hits[l], 4)})
            if flops[l] and share:
                # FC(h): flops of the live rows only (rows a partly filled tile pads do not count)
                per_layer[-1]["useful_TFLOPs"] = round(flops[l] / (share * 1e-3) / 1e12, 1)
            if n:
                k["bytes"] += algo[l]
                k["flops"] += flops[l]
                k["launches"] += 1
        if gbytes:
            k["ms"] += float(gms)
    # dominant kernel = the pooling instance that takes the most time in a pass
    dom_key = max(by_kernel, key=lambda kk: by_kernel[kk]["ms"])
    dom = by_kernel[dom_key]
    achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9 if dom["ms"] > 0 else 0.0
    roofline = {"bound": "hbm", "kernel": dom_key, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": PROFILED_TRAFFIC.get((name, dom_key), (None, None))[0],
                "traffic_source": PROFILED_TRAFFIC.get((name, dom_key), (None, None))[1],
                "bytes_per_launch": int(dom["bytes"] / max(1, dom["launches"])),
                "avg_launch_us": round(dom["ms"] / max(1, dom["launches"]) * 1e3, 2),
                "launches_per_step": dom["launches"]}
    if dom["flops"]:
        # FC(h): a dense contraction (split-K MFMA kernel + split reduction); report it against the
        # matrix-core peak of its dtype, and keep the byte rate beside it
        tf = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        peak = MFMA_PEAK_TFLOPS[spec.layers[0].dtype]
        roofline.update({"bound": "mfma", "achieved": round(tf, 1), "peak": peak, "unit": "TFLOP/s",
                         "frac": round(tf / peak, 4), "flops_per_launch": int(dom["flops"] / max(1, dom["launches"])),
                         "hbm_GBps": round(achieved, 1), "traffic": None, "traffic_source": None})
    pool_total_bytes = sum(k["bytes"] for k in by_kernel.values())
    pool_total_ms = sum(k["ms"] for k in by_kernel.values())
    out = {
        "workload": name, "ms_per_step": round(ms_step, 4), "wall_ms_per_step": round(wall_ms, 4),
        "lookups_per_step": lookups, "lookups_per_s": lookups / (ms_step * 1e-3),
        "request_layers_per_s": spec.batch * n_layers / (ms_step * 1e-3),
        "cumulative_hit_rate": round(1.0 - counts[n_layers] / spec.batch, 4),
        "pool_all_layers": {"GBps": round(pool_total_bytes / (pool_total_ms * 1e-3) / 1e9, 1),
                            "frac_of_peak": round(pool_total_bytes / (pool_total_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                            "us_per_step": round(pool_total_ms * 1e3, 1),
                            "share_of_step": round(pool_total_ms / ms_step, 3)},
        "roofline": roofline,
        "pool_kernels": {k: {"GBps": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] else 0.0,
                             "launches": v["launches"]} for k, v in by_kernel.items()},
        "layers": per_layer,
    }
    if spec.layers[0].predictor == "gap_mlp":
        pr = plain_read_same_sizes(spec, acts, counts, torch, g)
        out["pool_all_layers"]["plain_read_same_sizes_GBps"] = pr
        out["pool_all_layers"]["frac_of_plain_read_same_sizes"] = round(out["pool_all_layers"]["GBps"] / pr, 4) if pr else None
    out["head_us_per_step"] = round((ms_step - pool_total_ms) * 1e3, 1)     # FC layers, softmax, selector, finish + compaction
    out["compact_alone_us"] = time_compaction(caches[0], stack, spec.batch, torch)
    if graph:
        out["graph_ms_per_step"] = round(time_graph(stack, acts, steps, warmup, torch), 4)
    if overlap and spec.storage == "gather":
        out["overlap"] = time_overlap(stack, acts, steps, warmup, torch)
    if uncompacted and spec.storage == "gather":
        ms_all = time_uncompacted(spec, caches, acts, steps, warmup, torch)
        out["uncompacted"] = {"ms_per_step": round(ms_all, 4), "lookups_per_step": spec.batch * n_layers,
                              "requests_per_s": round(spec.batch / (ms_all * 1e-3), 1),
                              "requests_per_s_compacted": round(spec.batch / (ms_step * 1e-3), 1)}
    if ceiling:
        sc = stream_read_ceiling(acts, torch, g)
        out["stream_read_ceiling"] = sc
        out["roofline"]["frac_of_stream_read_ceiling"] = round(achieved / sc["GBps"], 4) if out["roofline"]["bound"] == "hbm" else None
        out["pool_all_layers"]["frac_of_stream_read_ceiling"] = round(out["pool_all_layers"]["GBps"] / sc["GBps"], 4)
        out["dependent_launch_floor"] = dependent_launch_floor(torch, g)
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(spec, weights, acts, stack, counts, cpu_requests, torch, W)
        if spec.storage == "gather":
            out["cpu_baseline_all_cores"] = cpu_baseline_all_cores(spec, weights, acts, cpu_requests, torch, W)
    if yardstick and spec.layers[0].predictor == "gap_mlp" and spec.storage == "gather":
        out["library_pool"] = pool_yardstick(spec, acts, torch)
    if train:
        out["train_step"] = time_training(spec, weights, caches, acts, torch, g, W, with_cpu)
    stack.close()
    del acts
    torch.cuda.empty_cache()
    return spec, out


def gemm_yardstick(spec, torch):
    """What the vendor GEMM behind torch.matmul reaches on this machine: on the layer-0 FC(h) product
    (random operands of the same shapes and dtype) and on a large square one."""
    def timed(fn, reps=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts.sort()
        return ts[len(ts) // 2] * 1e-3
    L = spec.layers[0]
    dt = torch.bfloat16 if L.dtype == "bf16" else torch.float32
    n, D, H = spec.batch, L.C * L.S, L.H
    x = torch.randn(n, D, device="cuda").clamp_(min=0).to(dt)
    w = torch.randn(H, D, device="cuda", dtype=torch.float32).to(dt)
    t1 = timed(lambda: x @ w.t())
    del x, w
    m = 8192
    a, b = torch.randn(m, m, device="cuda").to(dt), torch.randn(m, m, device="cuda").to(dt)
    t2 = timed(lambda: a @ b)
    return {"fc_shape": [n, D, H], "fc_us": round(t1 * 1e6, 1), "fc_TFLOPs": round(2.0 * n * D * H / t1 / 1e12, 1),
            "square_8192_us": round(t2 * 1e6, 1), "square_8192_TFLOPs": round(2.0 * m ** 3 / t2 / 1e12, 1)}


def conv_yardstick(spec, layers, torch):
    """The vendor convolution (torch conv2d + relu, NCHW as the library stores it) on random operands of
    one layer per map size, with that layer's active row count, beside this library's time for it."""
    out, seen = [], set()
    for l, L in enumerate(spec.layers):
        if L.in_hw in seen:
            continue
        seen.add(L.in_hw)
        n = max(1, int(layers[l]["n"]))
        dt = torch.bfloat16 if L.dtype == "bf16" else torch.float32
        k, s = L.conv_ks
        x = torch.randn(n, L.C, L.in_hw[0], L.in_hw[1], device="cuda").to(dt)
        w = torch.randn(L.H, L.C, k, k, device="cuda").to(dt)
        fn = lambda: torch.relu(torch.nn.functional.conv2d(x, w, stride=s))
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(10):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts.sort()
        out.append({"layer": l, "n": n, "C": L.C, "map": list(L.in_hw), "conv": [k, s], "filters": L.H,
                    "library_us": round(ts[len(ts) // 2] * 1e3, 1), "this_us": layers[l]["pool_us"]})
        del x, w
    return out


def time_training(spec, weights, caches, acts, torch, g, W, with_cpu, reps=10):
    """One retraining step (Section 5, "Retraining Learned Caches") per distinct cache shape of the
    workload, on a full batch: pooled features from the cache's own pooling kernel, then
    gati_trainer_step.  Context beside the lookup metric, not part of it."""
    n = spec.batch
    labels = W.zipf_labels(n, spec.layers[0].K, spec.zipf_s, spec.seed)
    Y = W.teacher_distribution(labels, spec.layers[0].K, spec.seed)
    lab_d, Y_d = torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda()
    out, seen = [], set()
    for l, L in enumerate(spec.layers):
        if (L.C, L.F) in seen:
            continue
        seen.add((L.C, L.F))
        pool_fc, fc_mlp, conv_fc = L.predictor == "pool_fc", L.predictor == "fc_mlp", L.predictor == "conv_fc"
        hid = L.sel_hidden if L.selector == "hidden" else 0
        F, Hd = L.F, (0 if pool_fc else L.H)
        if fc_mlp or conv_fc:
            # these predictors train on the activation itself: the rows as fp32 (the trainer's arithmetic)
            pooled = acts[l].reshape(n, -1).float()
        else:
            pooled = torch.empty((n, F), device="cuda")
            caches[l].pool(acts[l], None, n, None, pooled)
        tr = g.Trainer(L.C, Hd, L.K, weights[l], max_rows=n, sel_hidden=hid, predictor=L.predictor,
                       out_hw=getattr(L, "out_hw", (0, 0)), S=L.S, in_hw=getattr(L, "in_hw", (0, 0)),
                       conv_ks=getattr(L, "conv_ks", (0, 0)), selector=L.selector)
        losses = torch.zeros(2, device="cuda")
        for _ in range(3):
            tr.step(pooled, lab_d, Y_d, 0.002, 0.5, 2.0, losses)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(reps):
            tr.step(pooled, lab_d, Y_d, 0.002, 0.5, 2.0, losses)
        ev[1].record()
        torch.cuda.synchronize()
        us = ev[0].elapsed_time(ev[1]) / reps * 1e3
        # forward + backward products: predictor (3x the forward of each layer, the first layer's input gradient
        # is not needed), hidden-layer selector (forward + weight gradient)
        if fc_mlp:
            D = L.C * L.S
            flops = 4 * n * D * Hd + 6 * n * Hd * L.K
            Fs = Hd
        elif conv_fc:
            k = L.conv_ks[0]
            flops = 4 * n * F * L.C * k * k + 6 * n * F * L.K          # F = filters x positions
            Fs = F
        else:
            flops = (6 * n * Hd * L.K + 4 * n * F * Hd) if Hd else 4 * n * F * L.K
            Fs = F
        flops += 4 * n * (Fs + L.K) * hid
        row = {"layer": l, "predictor": L.predictor, "F": F, "H": Hd, "K": L.K, "selector_hidden": hid, "n": n,
               "step_us": round(us, 1), "TFLOPs": round(flops / (us * 1e-6) / 1e12, 2),
               "frac_of_fp32_mfma_peak": round(flops / (us * 1e-6) / 1e12 / 157.3, 4)}
        if fc_mlp:
            # the update streams the fp32 master copy of W1 once (read + write): the HBM floor of a step
            wb = 2 * Hd * L.C * L.S * 4
            row["W1_update_bytes"] = wb
            row["hbm_floor_us"] = round(wb / (HBM_PEAK_GBS * 1e9) * 1e6, 1)
        if conv_fc:
            # the convolution's two kernels run on the vector units: fp32 FMA without packed instructions,
            # 256 CUs x 64 lanes x 2 flop x 2.4 GHz
            row["bound"] = "alu"
            row["frac_of_fp32_vector_rate_unpacked"] = round(flops / (us * 1e-6) / 1e12 / 78.6, 4)
        if fc_mlp or conv_fc:
            out.append(row)
            tr.close()
            del pooled
            torch.cuda.empty_cache()
            continue
        if with_cpu and len(out) == 0:            # CPU baseline leg: the fp64 oracle's step on the same batch
            from oracle import train as otrain
            p_host = pooled.cpu().numpy()
            t0 = time.perf_counter()
            keys = (("W2", "b2") if pool_fc else ("W1", "b1", "W2", "b2")) + (("Ws", "cs", "vs") if hid else ("ws",)) + ("bs",)
            otrain.sgd_step({k: weights[l][k] for k in keys}, p_host, labels, Y, 0.002, 0.5, 2.0)
            row["oracle_cpu_ms"] = round((time.perf_counter() - t0) * 1e3, 1)
        out.append(row)
        tr.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50",
                    help="tiny | resnet18 | resnet50 | bert_base | resnet152")
    ap.add_argument("--also", default="bert_base,resnet18,resnet152,tiny",
                    help="comma-separated further workloads reported under 'others' ('' for none)")
    ap.add_argument("--cpu-requests", type=int, default=512,
                    help="requests of the batch the CPU oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", action="store_true", help="include the per-layer table in the JSON line")
    ap.add_argument("--graph", action="store_true", help="also time the pass replayed from a captured HIP graph")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the lookups beside a synthetic base-DNN stand-in, same stream vs side stream")
    ap.add_argument("--uncompacted", action="store_true",
                    help="also time the stack with every layer looking up the whole batch (no miss lists)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain tensor copy of layer 0's activations (known size), the reference "
                         "that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--library-yardstick", "--gemm-yardstick", dest="gemm_yardstick", action="store_true",
                    help="context, not a target: fc_mlp workloads also time the vendor GEMM (torch.matmul) on layer 0's "
                         "[n, D] x [D, H] and on a square 8192^3 product; conv_fc workloads time the vendor convolution "
                         "(torch conv2d + relu) on one layer of every map size; global-pool workloads time torch's mean "
                         "over the pooled axis of layer 0's tensor")
    ap.add_argument("--train", action="store_true",
                    help="also time one retraining step (gati_trainer_step, full batch) per distinct cache shape")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (one process, one MI355X); run it with --gpus 1. "
              "Requests are independent, so more GPUs would each run this same path on a share of the batch.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists for the product path)", file=sys.stderr)
        sys.exit(3)
    import paper_2101_07344_amd as g
    import workloads as W
    g.load_library()
    torch.cuda.set_device(0)

    stream = torch.cuda.Stream()          # default priority; every launch and event goes here
    with torch.cuda.stream(stream):
        spec, main_res = run_workload(args.workload, args.steps, args.warmup, not args.no_cpu_baseline,
                                      args.cpu_requests, torch, g, W, copy_probe=args.copy_probe,
                                      graph=args.graph, overlap=args.overlap, yardstick=args.gemm_yardstick,
                                      train=args.train, ceiling=True, uncompacted=args.uncompacted)
        others = {}
        for name in [n for n in args.also.split(",") if n and n != args.workload]:
            _, r = run_workload(name, args.steps, args.warmup, False, 0, torch, g, W)
            r.pop("layers", None)
            others[name] = r

    L0 = spec.layers[0]
    line = {
        "metric": "learned-cache lookups/sec (samples x layers)",
        "value": main_res["lookups_per_s"],
        "unit": "lookups/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": L0.dtype, "data": "synthetic",
        "config": {"workload": f"{spec.name}: batch {spec.batch}, {len(spec.layers)} caches, "
                               f"{L0.dtype} activations, storage {spec.storage}",
                   "lookups_per_step": main_res["lookups_per_step"],
                   "cumulative_hit_rate": main_res["cumulative_hit_rate"]},
        "roofline": main_res["roofline"],
        "cpu_baseline": main_res.get("cpu_baseline"),
        "cpu_baseline_all_cores": main_res.get("cpu_baseline_all_cores"),
        "stream_read_ceiling": main_res.get("stream_read_ceiling"),
        "request_layers_per_s": main_res["request_layers_per_s"],
        "pool_all_layers": main_res["pool_all_layers"],
        "pool_kernels": main_res["pool_kernels"],
        "others": others,
    }
    for key in ("head_us_per_step", "dependent_launch_floor", "compact_alone_us", "graph_ms_per_step", "overlap", "uncompacted", "library_pool", "train_step"):
        if key in main_res:
            line[key] = main_res[key]
    if args.gemm_yardstick and L0.predictor == "fc_mlp":
        line["library_gemm"] = gemm_yardstick(spec, torch)
    if args.gemm_yardstick and L0.predictor == "conv_fc":
        line["library_conv"] = conv_yardstick(spec, main_res["layers"], torch)
    if args.layers:
        line["layers"] = main_res["layers"]
    else:
        log(json.dumps(main_res["layers"]))
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
