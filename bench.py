#!/usr/bin/env python3
"""Benchmark of the message-passing hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Default workload `propagate` (the headline): the weighted-propagate-at-scale configuration (1 M nodes,
20 M directed edges from a seeded power-law multigraph, fp32 features F = 64), all inputs resident in
HBM before timing.  One step = one gnn_propagate(copy_xj, sum) over the whole graph; the
by-destination CSR is built once per graph, as a training loop reuses it across layers and epochs
(its build time and the other message/aggregation variants are reported under "extra").

Other workloads measure the remaining steps of the path, one JSON line each:
  csr      COO -> CSR build (range check, radix sort, degree histogram, scan, work lists) on the same graph
  temporal gnn_build_csr_batch on the same edge list cut into 8 snapshots, against 8 separate builds
  softmax  gnn_segment_softmax, 8 heads, on the same graph
  gcn      gnn_gcnconv on the 100 k-node / 1 M-edge symmetrised power-law graph, 128 -> 128 features
  gat      gnn_gatconv on the 2.45 M-node / 126 M-edge graph, 100 -> 8 heads x 8 channels
  gat_backward  gnn_gatconv_backward on the same graph
  batched  gnn_gin_update + gnn_graph_pool on 4 096 batched small graphs, F = 32
  tiny     gnn_propagate sum / mean / max on the 2 708-node graph (launch-latency bound)
  backward gnn_propagate_backward (e_mul_xj, sum: grad_x and grad_e) on the headline graph
  gcn_backward gnn_gcnconv_backward (grad X, W, b) on the GCN graph
  example  gnn_example_model_forward (the paper's example model) on collated batches of 32 and 4 096 graphs
  train    gnn_example_model_train_step (forward, loss, backward, Adam) on the same batches

Every line carries `value` (algorithmic GB/s = the byte model of the step / mean step time), a
`roofline` object for the dominant kernel and a `cpu_baseline` object (the parity oracle, one thread,
timed in the same run on a bounded sample).  Byte models are spelled out next to each workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E peak
MFMA_FP32_PEAK_TFLOPS = 157.3

# Hardware-counter figures of the dominant kernels come from profiles/counters.json: per-launch averages of separate
# `rocprofv3 --pmc` runs of this very file (commands and tables in the profiles/*.md named there).  A run of
# bench.py cannot read the counters itself; it attaches the stored figures only when workload, sizes and kernel
# name match, and null otherwise.  "traffic" = bytes that crossed the L2 <-> fabric boundary (read requests by
# size + write requests x 64 B); the Infinity Cache sits behind that boundary, so this is an upper bound of the
# HBM bytes, not the HBM bytes themselves (no counter on this part separates the two).
def load_counters():
    path = os.path.join(ROOT, "profiles", "counters.json")
    try:
        with open(path) as fh:
            return json.load(fh)
    except (OSError, ValueError):
        return {}


def counters_for(key):
    return load_counters().get(key)


def b_alg_propagate(n, e, f, e_dim=0):
    """One source row gathered per edge + neighbour id (+ edge data) + output rows + rowptr."""
    return e * (4 * f + 4 + 4 * e_dim) + n * 4 * f + (n + 1) * 4


def b_min_propagate(n, e, f, e_dim=0):
    """Every array touched exactly once."""
    return 2 * n * 4 * f + e * (4 + 4 * e_dim) + (n + 1) * 4


def time_calls(torch, fn, steps, warmup):
    """Mean milliseconds per call, HIP events on the stream the kernels are launched on."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / steps


def launch_distribution(torch, fn, launches=50, between=None):
    """Per-launch times (HIP events around every call): median, minimum and 95th percentile in milliseconds.
    `between` runs untimed before every launch (the cold regime: something that evicts the caches)."""
    for _ in range(3):
        fn()
    pairs = []
    for _ in range(launches):
        if between is not None:
            between()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in pairs)
    return {"median_ms": t[len(t) // 2], "min_ms": t[0], "p95_ms": t[min(len(t) - 1, int(0.95 * len(t)))],
            "launches": launches}


def streaming_probe(torch):
    """A plain streaming kernel (reads 1 GiB, writes 1 GiB): second denominator next to the spec-sheet
    peak, and the calibration dispatch for hardware-counter runs."""
    big = torch.zeros(256 * 1024 * 1024, dtype=torch.float32, device="cuda")
    big2 = torch.empty_like(big)
    ms = time_calls(torch, lambda: torch.add(big, 1.0, out=big2), 10, 2)
    return {"copy_kernel_GBs": 2 * big.numel() * 4 / (ms * 1e-3) / 1e9, "copy_kernel_bytes_each_way": big.numel() * 4}


def hbm_roofline(gbs, kernel, counters=None, seconds=None, b_min=None):
    """achieved / frac: algorithmic bytes per second (a gather rate: bytes served by the L2s count, so frac can
    exceed 1); frac_traffic: counter bytes beyond the L2s per second over the HBM peak (an upper bound of the HBM
    fraction); t_min_over_t: time the compulsory bytes would take at the HBM peak over the measured time."""
    r = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
         "traffic": None, "kernel": kernel}
    if b_min is not None and seconds:
        r["t_min_over_t"] = b_min / (HBM_PEAK_GBS * 1e9) / seconds
    if counters:
        r["traffic"] = counters.get("traffic_bytes")
        if seconds and counters.get("traffic_bytes"):
            r["frac_traffic"] = counters["traffic_bytes"] / seconds / 1e9 / HBM_PEAK_GBS
        for k in ("l2_read_hit_rate", "l2_read_requests", "fabric_read_requests", "source"):
            if k in counters:
                r[k] = counters[k]
    return r


def base_line(metric, gbs, ms, args, workload, config, dtype="f32"):
    cfg = {"workload": workload}
    cfg.update(config)
    return {"metric": metric, "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype,
            "data": "synthetic", "config": cfg}


def to_dev(torch, a):
    return torch.from_numpy(a).cuda()


# ----------------------------------------------------------------------------- workloads

def run_propagate(args, torch, gnn, synth):
    wl = synth.config2_weighted(num_nodes=args.nodes, num_edges=args.edges, feat=args.feat)
    n, e, f = wl.num_nodes, wl.num_edges, args.feat
    src, dst, x, ew = (to_dev(torch, a) for a in (wl.src, wl.dst, wl.x, wl.edge_weight))
    out = torch.empty_like(x)
    t0 = time.perf_counter()
    g = gnn.build_csr(src, dst, n)
    torch.cuda.synchronize()
    build_first_ms = (time.perf_counter() - t0) * 1e3

    ms = time_calls(torch, lambda: gnn.propagate(g, x, None, gnn.MSG_COPY_XJ, gnn.AGGR_SUM, out=out),
                    args.steps, args.warmup)
    bytes_alg = b_alg_propagate(n, e, f)
    gbs = bytes_alg / (ms * 1e-3) / 1e9
    extra = {"graph": wl.stats(), "work_lists": g.work_sizes(), "B_alg_bytes": bytes_alg,
             "B_min_bytes": b_min_propagate(n, e, f), "t_min_over_t": b_min_propagate(n, e, f) / 8e12 / (ms * 1e-3),
             "edge_feature_per_s": e * f / (ms * 1e-3), "csr_build_first_call_ms": build_first_ms}
    extra.update(streaming_probe(torch))
    if not args.no_extra:
        k = max(5, args.steps // 10)
        # warm = launches back to back; cold = 1 GiB streamed through the chip before every launch, which evicts
        # the L2s and the Infinity Cache (the graph's 0.6 GB working set does not fit them either way)
        headline = lambda: gnn.propagate(g, x, None, gnn.MSG_COPY_XJ, gnn.AGGR_SUM, out=out)
        extra["per_launch_warm"] = launch_distribution(torch, headline)
        evict_a = torch.zeros(256 * 1024 * 1024, dtype=torch.float32, device="cuda")
        evict_b = torch.empty_like(evict_a)
        extra["per_launch_cold"] = launch_distribution(torch, headline, between=lambda: torch.add(evict_a, 1.0, out=evict_b))
        del evict_a, evict_b
        e_csr = gnn.edge_data_to_csr(g, ew)
        for name, msg, aggr in (("e_mul_xj_sum", 1, 0), ("e_mul_xj_mean", 1, 1), ("e_mul_xj_max", 1, 2),
                                ("copy_xj_mean", 0, 1), ("copy_xj_max", 0, 2)):
            ed = e_csr if msg else None
            t = time_calls(torch, lambda: gnn.propagate(g, x, ed, msg, aggr, e_order=gnn.EDGE_ORDER_CSR, out=out), k, 3)
            extra[name] = {"ms": t, "GBs_alg": b_alg_propagate(n, e, f, msg) / (t * 1e-3) / 1e9}
        t = time_calls(torch, lambda: gnn.propagate(g, x, ew, 1, 0, e_order=gnn.EDGE_ORDER_COO, out=out), k, 3)
        extra["e_mul_xj_sum_coo_order"] = {"ms": t, "GBs_alg": b_alg_propagate(n, e, f, 1) / (t * 1e-3) / 1e9}
        if f % 8 == 0:
            # bfloat16 feature storage (widened exactly, float sums, float output): not the headline -- another
            # input precision -- reported to show what halving the gathered bytes buys
            xh = gnn.f32_to_bf16(x)
            for name, msg, aggr in (("bf16_storage_copy_xj_sum", 0, 0), ("bf16_storage_e_mul_xj_sum", 1, 0),
                                    ("bf16_storage_copy_xj_max", 0, 2)):
                ed = e_csr if msg else None
                t = time_calls(torch, lambda: gnn.propagate_bf16(g, xh, ed, msg, aggr, e_order=gnn.EDGE_ORDER_CSR, out=out), k, 3)
                b = e * (2 * f + 4 + 4 * msg) + n * 4 * f + (n + 1) * 4
                extra[name] = {"ms": t, "GBs_alg": b / (t * 1e-3) / 1e9, "edge_feature_per_s": e * f / (t * 1e-3)}
            del xh
            xh = gnn.f32_to_f16(x)      # IEEE binary16 storage: the same kernels with another widening
            t = time_calls(torch, lambda: gnn.propagate_f16(g, xh, None, 0, 0, out=out), k, 3)
            b = e * (2 * f + 4) + n * 4 * f + (n + 1) * 4
            extra["f16_storage_copy_xj_sum"] = {"ms": t, "GBs_alg": b / (t * 1e-3) / 1e9,
                                                "edge_feature_per_s": e * f / (t * 1e-3)}
            del xh
        extra["edge_data_to_csr_ms"] = time_calls(torch, lambda: gnn.edge_data_to_csr(g, ew), k, 2)
        # one float per edge through the two-pass route (gnn_graph_build_edge_route) instead of through perm
        csr_to_coo_direct = time_calls(torch, lambda: gnn.edge_data_to_coo(g, e_csr), k, 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.build_edge_route()
        torch.cuda.synchronize()
        route_build_ms = (time.perf_counter() - t0) * 1e3
        t_to_csr = time_calls(torch, lambda: gnn.edge_data_to_csr(g, ew), k, 2)
        t_to_coo = time_calls(torch, lambda: gnn.edge_data_to_coo(g, e_csr), k, 2)
        t = time_calls(torch, lambda: gnn.propagate(g, x, ew, 1, 0, e_order=gnn.EDGE_ORDER_COO, out=out), k, 3)
        extra["edge_route"] = {"build_ms": route_build_ms, "edge_data_to_csr_ms": t_to_csr,
                               "edge_data_to_coo_ms": t_to_coo, "edge_data_to_coo_direct_ms": csr_to_coo_direct,
                               "bytes_moved_per_direction": 24 * e, "GBs": 24 * e / (t_to_csr * 1e-3) / 1e9,
                               "e_mul_xj_sum_coo_order": {"ms": t, "GBs_alg": b_alg_propagate(n, e, f, 1) / (t * 1e-3) / 1e9}}
        gnn.build_csr(src, dst, n).close()      # steady state of a build-per-batch loop: arrays are reused from here on
        t0 = time.perf_counter()
        for _ in range(5):
            gnn.build_csr(src, dst, n).close()
        extra["csr_build_ms"] = (time.perf_counter() - t0) / 5 * 1e3
        extra["full_path_ms"] = extra["csr_build_ms"] + extra["edge_data_to_csr_ms"] + ms

    line = base_line("propagate(copy_xj,sum) algorithmic GB/s, 1M-node/20M-edge power-law graph, F=64", gbs, ms, args,
                     wl.name, {"N": n, "E": e, "F": f, "msg": "copy_xj", "aggr": "sum", "seed": synth.seed_of(2)})
    line["roofline"] = hbm_roofline(gbs, "propagate_kernel<16,4,0,0,0> = copy_xj, sum (+ combine_pieces_kernel, ~7 us)",
                                    counters_for(f"propagate:{n}:{e}:{f}"), ms * 1e-3, b_min_propagate(n, e, f))
    line["extra"] = extra
    if not args.no_cpu_baseline:
        import oracle
        es = min(args.cpu_sample_edges, e)
        t0 = time.perf_counter()
        oracle.propagate(wl.src[:es].copy(), wl.dst[:es].copy(), n, wl.x)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": b_alg_propagate(n, es, f) / dt / 1e9, "unit": "GB/s", "cores": 1,
                                "kind": "oracle", "seconds": dt, "edge_feature_per_s": es * f / dt,
                                "sample": f"copy_xj+sum over the first {es} of {e} edges (all {n} nodes, F={f}), one pass"}
        # the same sample with the oracle's rows dealt to all host cores (bit-identical result)
        t0 = time.perf_counter()
        _, threads = oracle.propagate_all_cores(wl.src[:es].copy(), wl.dst[:es].copy(), n, wl.x)
        dt = time.perf_counter() - t0
        line["cpu_baseline_all_cores"] = {"value": b_alg_propagate(n, es, f) / dt / 1e9, "unit": "GB/s",
                                          "cores": threads, "kind": "oracle, rows dealt to OpenMP threads",
                                          "seconds": dt, "edge_feature_per_s": es * f / dt,
                                          "sample": line["cpu_baseline"]["sample"]}
    g.close()
    return line


def run_csr(args, torch, gnn, synth):
    wl = synth.config2_weighted(num_nodes=args.nodes, num_edges=args.edges, feat=4)
    n, e = wl.num_nodes, wl.num_edges
    src, dst = to_dev(torch, wl.src), to_dev(torch, wl.dst)
    gnn.build_csr(src, dst, n).close()
    torch.cuda.synchronize()
    k = max(3, min(args.steps, 20))
    graphs = []
    t0 = time.perf_counter()
    for _ in range(k):
        graphs.append(gnn.build_csr(src, dst, n))     # synchronises internally
    ms = (time.perf_counter() - t0) / k * 1e3
    for g in graphs:
        g.close()
    # the loop of a training run: one graph per mini-batch, the previous one destroyed first (its arrays are reused)
    lib = gnn.lib()
    t0 = time.perf_counter()
    for _ in range(k):
        g = gnn.build_csr(src, dst, n)
        lib.gnn_graph_destroy(g._h)     # the build has synchronised: nothing is in flight
        g._h = None
    steady_ms = (time.perf_counter() - t0) / k * 1e3
    passes = max(1, ((max(n - 1, 1)).bit_length() + 7) // 8)
    # per pass: keys read twice (count + scatter) + two payloads read + three arrays written = 28 B/edge;
    # plus range check (8 B/edge), run detection (2 x 4 B/edge) and the row-sized scans and lists (~60 B/node)
    bytes_alg = e * (28 * passes + 16) + n * 60
    gbs = bytes_alg / (ms * 1e-3) / 1e9
    line = base_line("CSR-by-destination build, algorithmic GB/s (host wall clock per gnn_build_csr incl. allocations)",
                     gbs, ms, args, wl.name + ":csr_build", {"N": n, "E": e, "radix_passes": passes}, dtype="i32")
    line["steps"] = k
    line["roofline"] = hbm_roofline(gbs, "sort_scatter_kernel x%d dominates" % passes)
    line["extra"] = {"B_alg_bytes": bytes_alg, "edges_per_s": e / (ms * 1e-3),
                     "build_then_destroy_ms": steady_ms, "build_then_destroy_GBs_alg": bytes_alg / (steady_ms * 1e-3) / 1e9,
                     "note": "value: every build allocates its graph (handles kept alive); build_then_destroy: "
                             "the destroyed graph's arrays serve the next build"}
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.build_csr(wl.src, wl.dst, n)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": bytes_alg / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                "seconds": dt, "sample": "the whole edge list, one counting sort"}
    return line


def run_edge_data(args, torch, gnn, synth):
    """One float per edge from the caller's order into CSR order and back (gnn_edge_data_to_csr / _to_coo) on the
    headline graph: through perm directly, and through the two-pass route of gnn_graph_build_edge_route."""
    wl = synth.config2_weighted(num_nodes=args.nodes, num_edges=args.edges, feat=4)
    n, e = wl.num_nodes, wl.num_edges
    src, dst, ew = (to_dev(torch, a) for a in (wl.src, wl.dst, wl.edge_weight))
    g = gnn.build_csr(src, dst, n)
    k = max(5, min(args.steps, 50))
    e_csr = gnn.edge_data_to_csr(g, ew)
    direct_to_csr = time_calls(torch, lambda: gnn.edge_data_to_csr(g, ew), k, 3)
    direct_to_coo = time_calls(torch, lambda: gnn.edge_data_to_coo(g, e_csr), k, 3)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g.build_edge_route()
    torch.cuda.synchronize()
    route_build_ms = (time.perf_counter() - t0) * 1e3
    ms = time_calls(torch, lambda: gnn.edge_data_to_csr(g, ew), k, 3)
    ms_back = time_calls(torch, lambda: gnn.edge_data_to_coo(g, e_csr), k, 3)
    bytes_alg = 12 * e          # the value read, its index read, the value written
    gbs = bytes_alg / (ms * 1e-3) / 1e9
    line = base_line("edge data COO -> CSR order, one float per edge, algorithmic GB/s (12 bytes per edge)", gbs, ms,
                     args, wl.name + ":edge_data", {"N": n, "E": e, "e_dim": 1})
    line["steps"] = k
    line["roofline"] = hbm_roofline(gbs, "route_tile_forward_kernel + route_bucket_kernel<true>",
                                    counters_for(f"edge_data:{n}:{e}"), ms * 1e-3, bytes_alg)
    line["extra"] = {"B_alg_bytes": bytes_alg, "bytes_moved_by_the_route": 24 * e,
                     "route_GBs_moved": 24 * e / (ms * 1e-3) / 1e9, "to_coo_ms": ms_back,
                     "direct_to_csr_ms": direct_to_csr, "direct_to_coo_ms": direct_to_coo,
                     "route_build_ms": route_build_ms, "speedup_to_csr": direct_to_csr / ms}
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, n)
        w_h = np.ascontiguousarray(wl.edge_weight, dtype=np.float32).reshape(-1)
        t0 = time.perf_counter()
        w_h[perm]
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": bytes_alg / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                "seconds": dt, "sample": "e[perm] with the oracle's perm, all edges, one pass"}
    g.close()
    return line


def run_temporal(args, torch, gnn, synth):
    """Temporal snapshots: the headline edge list cut into 8 snapshots over the same nodes, built by one
    gnn_build_csr_batch call (one allocation, one synchronisation) and by 8 separate gnn_build_csr calls."""
    wl = synth.config2_weighted(num_nodes=args.nodes, num_edges=args.edges, feat=4)
    n, e = wl.num_nodes, wl.num_edges
    src, dst = to_dev(torch, wl.src), to_dev(torch, wl.dst)
    lib = gnn.lib()
    t_snap = 8
    cuts = [e * i // t_snap for i in range(t_snap + 1)]
    srcs = [src[cuts[i]:cuts[i + 1]] for i in range(t_snap)]
    dsts = [dst[cuts[i]:cuts[i + 1]] for i in range(t_snap)]

    def destroy(graphs):
        for g in graphs:
            lib.gnn_graph_destroy(g._h)     # the build has synchronised: nothing is in flight
            g._h = None

    destroy(gnn.build_csr_batch(srcs, dsts, n))
    k = max(3, min(args.steps, 10))
    t0 = time.perf_counter()
    for _ in range(k):
        destroy(gnn.build_csr_batch(srcs, dsts, n))
    ms = (time.perf_counter() - t0) / k * 1e3
    t0 = time.perf_counter()
    for _ in range(k):
        destroy([gnn.build_csr(a, b, n) for a, b in zip(srcs, dsts)])
    ms_sep = (time.perf_counter() - t0) / k * 1e3
    passes = max(1, ((max(n - 1, 1)).bit_length() + 7) // 8)
    bytes_alg = e * (28 * passes + 16) + t_snap * n * 60
    gbs = bytes_alg / (ms * 1e-3) / 1e9
    line = base_line("batch build of 8 snapshot graphs (gnn_build_csr_batch), algorithmic GB/s (host wall clock incl. allocation)",
                     gbs, ms, args, wl.name + ":temporal_batch_build", {"N": n, "E": e, "snapshots": t_snap}, dtype="i32")
    line["steps"] = k
    line["roofline"] = hbm_roofline(gbs, "sort_scatter_kernel on 2.5 M-edge snapshots dominates")
    line["extra"] = {"B_alg_bytes": bytes_alg, "separate_builds_ms": ms_sep,
                     "note": "the same 8 snapshots built by 8 gnn_build_csr calls take separate_builds_ms"}
    # the regime snapshot sequences are usually in: many small graphs.  256 snapshots of 20 000 edges over 10 000 nodes
    many, ne_small, n_small = 256, 20_000, 10_000
    s_src = [(src[i * ne_small:(i + 1) * ne_small] % n_small).contiguous() for i in range(many)]
    s_dst = [(dst[i * ne_small:(i + 1) * ne_small] % n_small).contiguous() for i in range(many)]
    destroy(gnn.build_csr_batch(s_src, s_dst, n_small))
    t0 = time.perf_counter()
    for _ in range(k):
        destroy(gnn.build_csr_batch(s_src, s_dst, n_small))
    ms_many = (time.perf_counter() - t0) / k * 1e3
    t0 = time.perf_counter()
    for _ in range(k):
        destroy([gnn.build_csr(a, b, n_small) for a, b in zip(s_src, s_dst)])
    ms_many_sep = (time.perf_counter() - t0) / k * 1e3
    line["extra"]["many_small_snapshots"] = {"snapshots": many, "N": n_small, "E_per_snapshot": ne_small,
                                             "batch_ms": ms_many, "separate_builds_ms": ms_many_sep}
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        for i in range(t_snap):
            oracle.build_csr(wl.src[cuts[i]:cuts[i + 1]], wl.dst[cuts[i]:cuts[i + 1]], n)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": bytes_alg / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                "seconds": dt, "sample": "all 8 snapshots, one counting sort each"}
    return line


def run_softmax(args, torch, gnn, synth):
    heads = 8
    wl = synth.config2_weighted(num_nodes=args.nodes, num_edges=args.edges, feat=4)
    n, e = wl.num_nodes, wl.num_edges
    g = gnn.build_csr(to_dev(torch, wl.src), to_dev(torch, wl.dst), n)
    s_host = (3.0 * synth.normal_f32(55, 2, e * heads)).reshape(e, heads)
    s = to_dev(torch, s_host)
    out = torch.empty_like(s)
    ms = time_calls(torch, lambda: gnn.segment_softmax(g, s, out=out), args.steps, args.warmup)
    # scores read twice, weights written once, perm + row id per edge for each pass, (max, den) per row and head
    bytes_alg = e * heads * 4 * 3 + e * 4 * 3 + n * heads * 8 * 2
    gbs = bytes_alg / (ms * 1e-3) / 1e9
    line = base_line("segment softmax (8 heads, COO-ordered scores) algorithmic GB/s", gbs, ms, args,
                     wl.name + ":segment_softmax", {"N": n, "E": e, "heads": heads})
    line["roofline"] = hbm_roofline(gbs, "normalise_kernel + stats kernels")
    line["extra"] = {"B_alg_bytes": bytes_alg, "edge_head_per_s": e * heads / (ms * 1e-3)}
    s_csr = gnn.edge_data_to_csr(g, s)
    t = time_calls(torch, lambda: gnn.segment_softmax(g, s_csr, order=gnn.EDGE_ORDER_CSR, out=out), max(5, args.steps // 4), 3)
    line["extra"]["csr_ordered_ms"] = t
    galpha = to_dev(torch, synth.normal_f32(55, 3, e * heads).reshape(e, heads))
    alpha = gnn.segment_softmax(g, s)
    gs = torch.empty_like(s)
    tb = time_calls(torch, lambda: gnn.segment_softmax_backward(g, alpha, galpha, out=gs), max(5, args.steps // 4), 3)
    line["extra"]["backward_ms"] = tb
    line["extra"]["backward_GBs_alg"] = (e * heads * 4 * 5 + e * 4 * 3 + n * heads * 8 * 2) / (tb * 1e-3) / 1e9
    del galpha, alpha, gs
    if not args.no_cpu_baseline:
        import oracle
        es = min(args.cpu_sample_edges, e)
        t0 = time.perf_counter()
        oracle.segment_softmax(wl.dst[:es].copy(), n, s_host[:es])
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": (es * heads * 12 + es * 12 + n * heads * 16) / dt / 1e9, "unit": "GB/s",
                                "cores": 1, "kind": "oracle", "seconds": dt,
                                "sample": f"the first {es} of {e} edges, 8 heads"}
    g.close()
    return line


def run_gcn(args, torch, gnn, synth):
    wl = synth.config1_gcn()
    n, e, f_in = wl.num_nodes, wl.num_edges, wl.x.shape[1]
    w_h, b_h = wl.params["w"], wl.params["bias"]
    f_out = w_h.shape[1]
    g = gnn.build_csr(to_dev(torch, wl.src), to_dev(torch, wl.dst), n)
    x, w, b = to_dev(torch, wl.x), to_dev(torch, w_h), to_dev(torch, b_h)
    out = torch.empty((n, f_out), dtype=torch.float32, device="cuda")
    ws = torch.empty(int(gnn.lib().gnn_gcnconv_workspace_bytes(n, f_out)), dtype=torch.uint8, device="cuda")
    ms = time_calls(torch, lambda: gnn.gcnconv(g, x, w, b, True, out=out, workspace=ws), args.steps, args.warmup)
    z = torch.empty_like(out)
    ms_xw = time_calls(torch, lambda: gnn.dense_xw(x, w, out=z), args.steps, args.warmup)
    ms_sp = time_calls(torch, lambda: gnn.gin_update(g, z, 0.0, out=out), args.steps, args.warmup)
    flops = 2.0 * n * f_in * f_out
    bytes_xw = 4 * (n * f_in + f_in * f_out + n * f_out)
    # sparse half: one Z row per edge and per (analytic) self-loop + ids + output + rowptr + degree factors
    bytes_sp = (e + n) * (4 * f_out + 4) + n * 4 * f_out + (n + 1) * 4 + n * 8
    gbs = (bytes_xw + bytes_sp) / (ms * 1e-3) / 1e9
    line = base_line("GCNConv forward (X W on MFMA + fused normalised SpMM) algorithmic GB/s", gbs, ms, args, wl.name,
                     {"N": n, "E": e, "f_in": f_in, "f_out": f_out, "add_self_loops": True})
    b_min_sp = 2 * n * 4 * f_out + e * 4 + (n + 1) * 4 + n * 8
    line["roofline"] = hbm_roofline(bytes_sp / (ms_sp * 1e-3) / 1e9,
                                    "propagate_kernel<32,4,copy_xj,sum> with GCN epilogue (timed alone through "
                                    "gnn_gin_update on Z: same gathers, same epilogue shape)",
                                    counters_for(f"gcn:{n}:{e}:{f_out}"), ms_sp * 1e-3, b_min_sp)
    line["extra"] = {"graph": wl.stats(), "xw_ms": ms_xw, "spmm_ms": ms_sp, "B_alg_spmm_bytes": bytes_sp,
                     "xw_roofline": {"bound": "mfma", "achieved": flops / (ms_xw * 1e-3) / 1e12,
                                     "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": flops / (ms_xw * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS,
                                     "hbm_GBs": bytes_xw / (ms_xw * 1e-3) / 1e9, "kernel": "xw_fast_kernel<NT=1,KQ=4> (32-column tiles, four k quarters)"}}
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.gcnconv(wl.src, wl.dst, n, wl.x, w_h, b_h, True)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": (bytes_xw + bytes_sp) / dt / 1e9, "unit": "GB/s", "cores": 1,
                                "kind": "oracle", "seconds": dt, "sample": "the whole layer, one pass"}
    g.close()
    return line


def run_gat(args, torch, gnn, synth):
    wl = synth.config4_gat()
    p = wl.params
    n, e, f_in = wl.num_nodes, wl.num_edges, wl.x.shape[1]
    heads, ch = p["heads"], p["ch"]
    hc = heads * ch
    g = gnn.build_csr(to_dev(torch, wl.src), to_dev(torch, wl.dst), n)
    x, w, a_s, a_d = (to_dev(torch, a) for a in (wl.x, p["w"], p["a_src"], p["a_dst"]))
    out = torch.empty((n, hc), dtype=torch.float32, device="cuda")
    ws = torch.empty(int(gnn.lib().gnn_gatconv_workspace_bytes(n, heads, ch)), dtype=torch.uint8, device="cuda")
    steps = max(3, min(args.steps, 30))
    ms = time_calls(torch, lambda: gnn.gatconv(g, x, w, a_s, a_d, 0.2, out=out, workspace=ws), steps, 3)
    h = torch.empty_like(out)
    ms_xw = time_calls(torch, lambda: gnn.dense_xw(x, w, out=h), steps, 3)
    flops = 2.0 * n * f_in * hc
    bytes_xw = 4 * (n * f_in + f_in * hc + n * hc)
    # attention pass: per edge one h row + its source scores + neighbour id; per node output, both score rows, rowptr
    bytes_att = e * (4 * hc + 4 * heads + 4) + n * (4 * hc + 8 * heads + 4) + n * 4 * hc + n * 8 * heads
    ms_att = ms - ms_xw
    gbs = (bytes_xw + bytes_att) / (ms * 1e-3) / 1e9
    line = base_line("GAT layer forward (X W on MFMA + fused score/softmax/aggregate) algorithmic GB/s", gbs, ms, args,
                     wl.name, {"N": n, "E": e, "f_in": f_in, "heads": heads, "ch": ch})
    line["steps"] = steps
    b_min_att = 2 * n * 4 * hc + e * 4 + n * (8 * heads + 4)
    line["roofline"] = hbm_roofline(bytes_att / (ms_att * 1e-3) / 1e9,
                                    "gat_kernel<16,4,2> (+ node_scores_kernel, gat_merge_kernel); time = layer - X W",
                                    counters_for(f"gat:{n}:{e}:{hc}"), ms_att * 1e-3, b_min_att)
    line["extra"] = {"xw_ms": ms_xw, "attention_ms": ms_att, "B_alg_attention_bytes": bytes_att,
                     "edge_feature_per_s": e * hc / (ms_att * 1e-3), "work_lists": g.work_sizes(),
                     "xw_roofline": {"bound": "mfma", "achieved": flops / (ms_xw * 1e-3) / 1e12,
                                     "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": flops / (ms_xw * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS,
                                     "hbm_GBs": bytes_xw / (ms_xw * 1e-3) / 1e9, "kernel": "xw_fast_kernel<NT=2,KQ=4> (64-column tiles, k = 100 in 3 full quarters + 2 k-steps)"}}
    if not args.no_cpu_baseline:
        import oracle
        es = min(args.cpu_sample_edges // 4, e)        # a prefix of the edge list over a node prefix
        ns = min(n, 200_000)
        m = (wl.src[:es] < ns) & (wl.dst[:es] < ns)
        s_src, s_dst = wl.src[:es][m].copy(), wl.dst[:es][m].copy()
        t0 = time.perf_counter()
        oracle.gatconv(s_src, s_dst, ns, wl.x[:ns], p["w"], p["a_src"], p["a_dst"], 0.2)
        dt = time.perf_counter() - t0
        ee = int(s_src.shape[0])
        b = 4 * (ns * f_in + f_in * hc + ns * hc) + ee * (4 * hc + 4 * heads + 4) + ns * (8 * hc + 16 * heads + 4)
        line["cpu_baseline"] = {"value": b / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle", "seconds": dt,
                                "sample": f"the layer on the first {ns} nodes and the {ee} edges among them"}
    g.close()
    return line


def run_gat_backward(args, torch, gnn, synth):
    wl = synth.config4_gat()
    p = wl.params
    n, e, f_in = wl.num_nodes, wl.num_edges, wl.x.shape[1]
    heads, ch = p["heads"], p["ch"]
    hc = heads * ch
    src, dst = to_dev(torch, wl.src), to_dev(torch, wl.dst)
    g, gt = gnn.build_csr(src, dst, n), gnn.build_csr(dst, src, n)
    del src, dst
    x, w, a_s, a_d = (to_dev(torch, a) for a in (wl.x, p["w"], p["a_src"], p["a_dst"]))
    gout_h = synth.normal_f32(47, 7, n * hc).reshape(n, hc)
    gout = to_dev(torch, gout_h)
    stats = torch.empty((n, heads, 2), dtype=torch.float32, device="cuda")
    out = gnn.gatconv(g, x, w, a_s, a_d, 0.2, softmax_stats=stats)
    ws = torch.empty(int(gnn.lib().gnn_gatconv_backward_workspace_bytes(n, f_in, heads, ch)), dtype=torch.uint8,
                     device="cuda")
    steps = max(3, min(args.steps, 20))
    ms = time_calls(torch, lambda: gnn.gatconv_backward(g, gt, x, w, a_s, a_d, out, stats, gout, 0.2, workspace=ws),
                    steps, 2)
    # two edge passes: each gathers one feature row and the scalars of the other endpoint per edge
    bytes_dst_pass = e * (4 * hc + 4 * heads + 4) + n * (4 * hc + 16 * heads + 4 * heads + 4)
    bytes_src_pass = e * (4 * hc + 16 * heads + 4) + n * (8 * hc + 4 * heads + 4 * heads + 4)
    bytes_dense = 3 * 4 * (n * f_in + f_in * hc + n * hc) + 6 * 4 * n * hc   # X W, dh W^T, X^T dh; records, score terms
    gbs = (bytes_dst_pass + bytes_src_pass + bytes_dense) / (ms * 1e-3) / 1e9
    line = base_line("GAT layer backward (grad X, W, a_src, a_dst) algorithmic GB/s", gbs, ms, args,
                     wl.name + ":backward", {"N": n, "E": e, "f_in": f_in, "heads": heads, "ch": ch})
    line["steps"] = steps
    line["roofline"] = hbm_roofline(gbs, "whole call; dominated by gat_backward_kernel<16,4,false> and <16,4,true>")
    line["extra"] = {"B_alg_dst_pass_bytes": bytes_dst_pass, "B_alg_src_pass_bytes": bytes_src_pass,
                     "B_alg_dense_bytes": bytes_dense, "work_lists_by_source": gt.work_sizes()}
    if not args.no_cpu_baseline:
        import oracle
        es = min(args.cpu_sample_edges, e)
        ns = min(n, 200_000)
        m = (wl.src[:es] < ns) & (wl.dst[:es] < ns)
        s_src, s_dst = wl.src[:es][m].copy(), wl.dst[:es][m].copy()
        t0 = time.perf_counter()
        oracle.gatconv_backward(s_src, s_dst, ns, wl.x[:ns], p["w"], p["a_src"], p["a_dst"], gout_h[:ns], 0.2)
        dt = time.perf_counter() - t0
        ee = int(s_src.shape[0])
        b = (ee * (8 * hc + 20 * heads + 8) + ns * (12 * hc + 32 * heads) +
             3 * 4 * (ns * f_in + f_in * hc + ns * hc) + 6 * 4 * ns * hc)
        line["cpu_baseline"] = {"value": b / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle", "seconds": dt,
                                "sample": f"the backward on the first {ns} nodes and the {ee} edges among them"}
    g.close()
    gt.close()
    return line


def run_example(args, torch, gnn, synth):
    """The paper's example model, forward, on a collated batch: 32 graphs (the listing's batch size) and 4 096."""
    results = {}
    for ng in (32, 4096):
        wl = synth.config5_example_model(num_graphs=ng)
        n, e, p = wl.num_nodes, wl.num_edges, wl.params
        g = gnn.build_csr(to_dev(torch, wl.src), to_dev(torch, wl.dst), n)
        x, gi = to_dev(torch, wl.x), to_dev(torch, wl.graph_indicator)
        dp = {k: to_dev(torch, v) for k, v in p.items()}
        f0, f1, f2, f3 = wl.x.shape[1], p["w1"].shape[1], p["w2"].shape[1], p["w3"].shape[1]
        y = torch.empty((ng, f3), dtype=torch.float32, device="cuda")
        ws = torch.empty(int(gnn.lib().gnn_example_model_workspace_bytes(n, ng, f1, f2)), dtype=torch.uint8, device="cuda")
        ms = time_calls(torch, lambda: gnn.example_model_forward(g, gi, ng, x, dp, out=y, workspace=ws), args.steps,
                        args.warmup)
        # per layer: GCN = X read, Z written and gathered (E + N rows), output written; batch norm reads its
        # input three times and writes once; pooling reads h3; plus indices
        b = (4 * n * (f0 + 2 * f1) + (e + n) * (4 * f1 + 4) + 4 * 4 * n * f1 +
             4 * n * (f1 + 2 * f2) + (e + n) * (4 * f2 + 4) + 4 * n * f2 + 4 * n)
        # the same call captured once into a HIP graph and replayed (the chain is ~20 small launches)
        gph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gph):
            gnn.example_model_forward(g, gi, ng, x, dp, out=y, workspace=ws)
        ms_graph = time_calls(torch, gph.replay, args.steps, args.warmup)
        results[ng] = (ms, b, n, e, ms_graph)
        del gph
        g.close()
    ms, b, n, e, ms_graph = results[4096]
    line = base_line("example model forward (GCNConv, BatchNorm, relu, GCNConv+relu, mean pool, Dense), algorithmic GB/s",
                     b / (ms * 1e-3) / 1e9, ms, args, "config5_example_model:4096_graphs",
                     {"graphs": 4096, "N": n, "E": e, "widths": "16-64-64-1"})
    line["roofline"] = hbm_roofline(b / (ms * 1e-3) / 1e9, "whole chain (9 dependent launches)")
    line["extra"] = {"graphs_per_s": 4096 / (ms * 1e-3), "batch_of_32_graphs_ms": results[32][0],
                     "batch_of_32_graphs_per_s": 32 / (results[32][0] * 1e-3),
                     "hip_graph_replay_ms": ms_graph, "batch_of_32_hip_graph_replay_ms": results[32][4],
                     "note": "the batch of 32 graphs (1 600 nodes) is launch-latency bound"}
    if not args.no_cpu_baseline:
        import oracle
        wl = synth.config5_example_model(num_graphs=4096)
        t0 = time.perf_counter()
        oracle.example_model_forward(wl.src, wl.dst, wl.num_nodes, wl.graph_indicator, 4096, wl.x, wl.params)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": b / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle", "seconds": dt,
                                "sample": "the whole batch of 4 096 graphs, one pass"}
    return line


def run_train(args, torch, gnn, synth):
    """One training step of the paper's example model (forward, MSE loss, all gradients, Adam) per call."""
    results = {}
    for ng in (32, 4096):
        wl = synth.config5_example_model(num_graphs=ng)
        n, e, p = wl.num_nodes, wl.num_edges, wl.params
        src, dst = to_dev(torch, wl.src), to_dev(torch, wl.dst)
        g, gt = gnn.build_csr(src, dst, n), gnn.build_csr(dst, src, n)
        x, gi = to_dev(torch, wl.x), to_dev(torch, wl.graph_indicator)
        target = to_dev(torch, synth.normal_f32(95, 9, ng).reshape(ng, 1))
        dp = {k: to_dev(torch, v) for k, v in p.items()}
        dm = {k: torch.zeros_like(v) for k, v in dp.items()}
        dv = {k: torch.zeros_like(v) for k, v in dp.items()}
        f0, f1, f2, f3 = wl.x.shape[1], p["w1"].shape[1], p["w2"].shape[1], p["w3"].shape[1]
        ws = torch.empty(int(gnn.lib().gnn_example_model_train_workspace_bytes(n, ng, f0, f1, f2, f3)), dtype=torch.uint8,
                         device="cuda")
        loss = torch.empty(1, dtype=torch.float32, device="cuda")
        counter = [0]

        def step():
            counter[0] += 1
            gnn.example_model_train_step(g, gt, gi, ng, x, target, dp, dm, dv, counter[0], loss=loss, workspace=ws)

        ms = time_calls(torch, step, args.steps, args.warmup)
        results[ng] = (ms, n, e, float(loss.cpu()[0]))
        g.close()
        gt.close()
    ms, n, e, last_loss = results[4096]
    f1 = f2 = 64
    # forward bytes (see the example workload) + backward: two GCN backward passes, batch-norm backward, masks
    b_fwd = (4 * n * (16 + 2 * f1) + (e + n) * (4 * f1 + 4) + 4 * 4 * n * f1 + 4 * n * (f1 + 2 * f2) + (e + n) * (4 * f2 + 4) +
             4 * n * f2 + 4 * n)
    b_bwd = 2 * ((e + n) * (4 * f1 + 4) + 6 * 4 * n * f1) + 5 * 4 * n * f1 + 3 * 4 * n * f2
    line = base_line("example model training step (forward, MSE, backward, Adam), algorithmic GB/s",
                     (b_fwd + b_bwd) / (ms * 1e-3) / 1e9, ms, args, "config5_example_model:train:4096_graphs",
                     {"graphs": 4096, "N": n, "E": e, "widths": "16-64-64-1", "optimizer": "Adam(1e-4)"})
    line["roofline"] = hbm_roofline((b_fwd + b_bwd) / (ms * 1e-3) / 1e9, "whole step (about 35 dependent launches)")
    line["extra"] = {"graphs_per_s": 4096 / (ms * 1e-3), "steps_per_s": 1e3 / ms, "loss_after_timed_steps": last_loss,
                     "batch_of_32_graphs_ms": results[32][0], "batch_of_32_steps_per_s": 1e3 / results[32][0]}
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        wl = synth.config5_example_model(num_graphs=4096)
        target = synth.normal_f32(95, 9, 4096).reshape(4096, 1)
        t0 = time.perf_counter()
        _, grads, _ = oracle.example_model_backward(wl.src, wl.dst, wl.num_nodes, wl.graph_indicator, 4096, wl.x, wl.params,
                                                    target)
        for k, v in wl.params.items():
            oracle.adam_step(v, np.zeros_like(v), np.zeros_like(v), grads[k], 1e-4, 1)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": (b_fwd + b_bwd) / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                "seconds": dt, "sample": "one whole training step on the batch of 4 096 graphs"}
    return line


def run_batched(args, torch, gnn, synth):
    wl = synth.config3_batched()
    n, e, f, ng = wl.num_nodes, wl.num_edges, wl.x.shape[1], wl.num_graphs
    g = gnn.build_csr(to_dev(torch, wl.src), to_dev(torch, wl.dst), n)
    x, gi = to_dev(torch, wl.x), to_dev(torch, wl.graph_indicator)
    upd = torch.empty_like(x)
    pooled = torch.empty((ng, f), dtype=torch.float32, device="cuda")

    def step():
        gnn.gin_update(g, x, 0.0, out=upd)
        gnn.graph_pool(gi, ng, upd, gnn.AGGR_SUM, out=pooled)

    ms = time_calls(torch, step, args.steps, args.warmup)
    ms_gin = time_calls(torch, lambda: gnn.gin_update(g, x, 0.0, out=upd), args.steps, args.warmup)
    ms_pool = time_calls(torch, lambda: gnn.graph_pool(gi, ng, upd, gnn.AGGR_SUM, out=pooled), args.steps, args.warmup)
    bytes_gin = e * (4 * f + 4) + 3 * n * 4 * f + (n + 1) * 4
    bytes_pool = n * 4 * f + n * 4 + ng * 4 * f
    gbs = (bytes_gin + bytes_pool) / (ms * 1e-3) / 1e9
    line = base_line("GIN update + sum pooling on 4096 batched small graphs, algorithmic GB/s", gbs, ms, args, wl.name,
                     {"N": n, "E": e, "F": f, "graphs": ng})
    line["roofline"] = hbm_roofline(bytes_gin / (ms_gin * 1e-3) / 1e9, "propagate_kernel<8,4,copy_xj,sum> with self term")
    line["extra"] = {"gin_ms": ms_gin, "pool_ms": ms_pool, "pool_GBs": bytes_pool / (ms_pool * 1e-3) / 1e9,
                     "note": "the whole problem (13 MB of features) fits the caches: launch latency dominates"}
    if not args.no_extra:
        # the other end of pooling: few, large graphs (one graph of 1 M nodes, 8 graphs of 125 000 nodes), F = 64 --
        # one block per graph (gnn_graph_pool) against several blocks per graph (gnn_graph_pool_ws)
        big_n, big_f = 1_000_000, 64
        xb = torch.randn((big_n, big_f), dtype=torch.float32, device="cuda")
        big = {}
        for graphs in (1, 8):
            gib = (torch.arange(big_n, device="cuda") // (big_n // graphs)).clamp(max=graphs - 1).to(torch.int32)
            ob = torch.empty((graphs, big_f), dtype=torch.float32, device="cuda")
            wsb = torch.empty(int(gnn.lib().gnn_graph_pool_workspace_bytes(big_n, graphs, big_f)), dtype=torch.uint8,
                              device="cuda")
            t_ws = time_calls(torch, lambda: gnn.graph_pool_ws(gib, graphs, xb, gnn.AGGR_SUM, out=ob, workspace=wsb), 20, 3)
            t_one = time_calls(torch, lambda: gnn.graph_pool(gib, graphs, xb, gnn.AGGR_SUM, out=ob), 3, 1)
            big[f"{graphs}_graphs"] = {"pool_ws_ms": t_ws, "pool_ms": t_one,
                                       "pool_ws_GBs": big_n * big_f * 4 / (t_ws * 1e-3) / 1e9}
        line["extra"]["large_graphs_1M_nodes_F64"] = big
        del xb
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        u = oracle.gin_update(wl.src, wl.dst, n, wl.x, 0.0)
        oracle.graph_pool(wl.graph_indicator, ng, u)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": (bytes_gin + bytes_pool) / dt / 1e9, "unit": "GB/s", "cores": 1,
                                "kind": "oracle", "seconds": dt, "sample": "the whole batch, one pass"}
    g.close()
    return line


def run_tiny(args, torch, gnn, synth):
    wl = synth.config0_tiny()
    n, e, f = wl.num_nodes, wl.num_edges, wl.x.shape[1]
    g = gnn.build_csr(to_dev(torch, wl.src), to_dev(torch, wl.dst), n)
    x = to_dev(torch, wl.x)
    out = torch.empty_like(x)
    times = {}
    for name, aggr in (("sum", 0), ("mean", 1), ("max", 2)):
        times[name] = time_calls(torch, lambda: gnn.propagate(g, x, None, 0, aggr, out=out), args.steps, args.warmup)
    ms = times["sum"]
    bytes_alg = b_alg_propagate(n, e, f)
    gbs = bytes_alg / (ms * 1e-3) / 1e9
    line = base_line("tiny propagate (2708 nodes): algorithmic GB/s (launch-latency bound; see us_per_call)", gbs, ms,
                     args, wl.name, {"N": n, "E": e, "F": f})
    line["roofline"] = hbm_roofline(gbs, "propagate_kernel<16,4,copy_xj,sum>")
    line["extra"] = {"us_per_call": {k: v * 1e3 for k, v in times.items()}}
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        reps = 200
        for _ in range(reps):
            oracle.propagate(wl.src, wl.dst, n, wl.x)
        dt = (time.perf_counter() - t0) / reps
        line["cpu_baseline"] = {"value": bytes_alg / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                "seconds": dt, "sample": "the whole graph, mean of 200 passes"}
    g.close()
    return line


def run_backward(args, torch, gnn, synth):
    wl = synth.config2_weighted(num_nodes=args.nodes, num_edges=args.edges, feat=args.feat)
    n, e, f = wl.num_nodes, wl.num_edges, args.feat
    src, dst, x, ew = (to_dev(torch, a) for a in (wl.src, wl.dst, wl.x, wl.edge_weight))
    g = gnn.build_csr(src, dst, n)
    gt = gnn.build_csr(dst, src, n)      # the same edges sorted by source
    gout_h = synth.normal_f32(17, 7, n * f).reshape(n, f)
    gout = to_dev(torch, gout_h)
    steps = max(5, args.steps // 4)
    ms = time_calls(torch, lambda: gnn.propagate_backward(g, gt, x, gout, ew, gnn.MSG_E_MUL_XJ, gnn.AGGR_SUM), steps, 3)
    ms_x = time_calls(torch, lambda: gnn.propagate_backward(g, gt, x, gout, ew, gnn.MSG_E_MUL_XJ, gnn.AGGR_SUM,
                                                            want_grad_e=False), steps, 3)
    ms_e = time_calls(torch, lambda: gnn.propagate_backward(g, gt, x, gout, ew, gnn.MSG_E_MUL_XJ, gnn.AGGR_SUM,
                                                            want_grad_x=False), steps, 3)
    # grad_x: a propagate over the by-source graph with weights fetched through perm;
    # grad_e: two feature rows, three indices and one result per edge
    bytes_x = e * (4 * f + 4 + 4 + 4) + n * 4 * f + (n + 1) * 4
    bytes_e = e * (8 * f + 12 + 4)
    gbs = (bytes_x + bytes_e) / (ms * 1e-3) / 1e9
    line = base_line("backward of propagate(e_mul_xj, sum): grad_x and grad_e, algorithmic GB/s", gbs, ms, args,
                     wl.name + ":backward", {"N": n, "E": e, "F": f, "msg": "e_mul_xj", "aggr": "sum"})
    line["steps"] = steps
    line["roofline"] = hbm_roofline(bytes_x / (ms_x * 1e-3) / 1e9, "propagate_kernel<16,4,e_mul_xj,sum> on the by-source graph")
    line["extra"] = {"grad_x_ms": ms_x, "grad_e_ms": ms_e, "grad_e_GBs": bytes_e / (ms_e * 1e-3) / 1e9,
                     "B_alg_grad_x_bytes": bytes_x, "B_alg_grad_e_bytes": bytes_e}
    # the same calls when both graphs carry a route for one float per edge: the weights reach the by-source pass
    # and the edge gradients leave the by-destination pass in streams instead of through perm
    g.build_edge_route()
    gt.build_edge_route()
    r_ms = time_calls(torch, lambda: gnn.propagate_backward(g, gt, x, gout, ew, gnn.MSG_E_MUL_XJ, gnn.AGGR_SUM), steps, 3)
    r_x = time_calls(torch, lambda: gnn.propagate_backward(g, gt, x, gout, ew, gnn.MSG_E_MUL_XJ, gnn.AGGR_SUM,
                                                           want_grad_e=False), steps, 3)
    r_e = time_calls(torch, lambda: gnn.propagate_backward(g, gt, x, gout, ew, gnn.MSG_E_MUL_XJ, gnn.AGGR_SUM,
                                                           want_grad_x=False), steps, 3)
    line["extra"]["with_edge_route"] = {"ms": r_ms, "grad_x_ms": r_x, "grad_e_ms": r_e,
                                        "GBs_alg": (bytes_x + bytes_e) / (r_ms * 1e-3) / 1e9}
    if not args.no_cpu_baseline:
        import oracle
        es = min(args.cpu_sample_edges // 2, e)
        t0 = time.perf_counter()
        oracle.propagate_backward(wl.src[:es].copy(), wl.dst[:es].copy(), n, wl.x, gout_h, wl.edge_weight[:es].copy(),
                                  1, 0)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": (es * (12 * f + 28) + n * 4 * f) / dt / 1e9, "unit": "GB/s", "cores": 1,
                                "kind": "oracle", "seconds": dt, "sample": f"the first {es} of {e} edges, one pass"}
    g.close()
    gt.close()
    return line


def run_gcn_backward(args, torch, gnn, synth):
    wl = synth.config1_gcn()
    n, e, f_in = wl.num_nodes, wl.num_edges, wl.x.shape[1]
    w_h = wl.params["w"]
    f_out = w_h.shape[1]
    src, dst = to_dev(torch, wl.src), to_dev(torch, wl.dst)
    g, gt = gnn.build_csr(src, dst, n), gnn.build_csr(dst, src, n)
    x, w = to_dev(torch, wl.x), to_dev(torch, w_h)
    gout_h = synth.normal_f32(33, 7, n * f_out).reshape(n, f_out)
    gout = to_dev(torch, gout_h)
    ws = torch.empty(int(gnn.lib().gnn_gcnconv_backward_workspace_bytes(n, f_in, f_out)), dtype=torch.uint8, device="cuda")
    ms = time_calls(torch, lambda: gnn.gcnconv_backward(g, gt, x, w, gout, True, workspace=ws), args.steps, args.warmup)
    # T = Ahat^T G (a GCN sparse half on G), T W^T and X^T T (each reads two N x f matrices and W), column sums
    bytes_sp = (e + n) * (4 * f_out + 4) + 3 * n * 4 * f_out + (n + 1) * 4 + n * 8
    bytes_dense = 4 * (n * f_out + f_in * f_out + n * f_in) + 4 * (n * f_in + n * f_out + f_in * f_out) + 4 * n * f_out
    flops = 4.0 * n * f_in * f_out
    gbs = (bytes_sp + bytes_dense) / (ms * 1e-3) / 1e9
    line = base_line("GCNConv backward (grad X, W, b) algorithmic GB/s", gbs, ms, args, wl.name + ":backward",
                     {"N": n, "E": e, "f_in": f_in, "f_out": f_out})
    line["roofline"] = hbm_roofline(gbs, "whole call: propagate_kernel<32,4> on the by-source graph, xw_fast_kernel, "
                                         "xty_partial_kernel, reductions")
    line["extra"] = {"dense_flops": flops, "dense_TFLOPs_if_all_time_were_dense": flops / (ms * 1e-3) / 1e12}
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.gcnconv_backward(wl.src, wl.dst, n, wl.x, w_h, gout_h, True)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": (bytes_sp + bytes_dense) / dt / 1e9, "unit": "GB/s", "cores": 1,
                                "kind": "oracle", "seconds": dt, "sample": "the whole layer, one pass"}
    g.close()
    gt.close()
    return line


WORKLOADS = {"edge_data": run_edge_data, "temporal": run_temporal, "train": run_train, "example": run_example, "gat_backward": run_gat_backward, "gcn_backward": run_gcn_backward, "backward": run_backward, "propagate": run_propagate, "csr": run_csr, "softmax": run_softmax, "gcn": run_gcn, "gat": run_gat,
             "batched": run_batched, "tiny": run_tiny}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="propagate")
    ap.add_argument("--nodes", type=int, default=1_000_000)
    ap.add_argument("--edges", type=int, default=20_000_000)
    ap.add_argument("--feat", type=int, default=64)
    ap.add_argument("--cpu-sample-edges", type=int, default=20_000_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="time only the headline step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2412_06354_amd import binding as gnn, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    gnn.lib()    # raises if the HIP library has not been built
    torch.cuda.set_device(0)
    print(json.dumps(WORKLOADS[args.workload](args, torch, gnn, synth)))


if __name__ == "__main__":
    main()
