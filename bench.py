#!/usr/bin/env python3
"""Benchmark of the propagate hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: the weighted-propagate-at-scale configuration (1 M nodes, 20 M directed edges from a
seeded power-law multigraph, fp32 features F = 64), all inputs resident in HBM before timing.
One step = one gnn_propagate(copy_xj, sum) over the whole graph (the by-destination CSR is built
once per graph, as a training loop reuses it across layers and epochs; its build time and the
other message/aggregation variants are reported in the same line under "extra").

Prints ONE JSON line.  value = algorithmic GB/s of the step:
  B_alg = E*(4F + 4) + N*4F + (N+1)*4  bytes  (one source row gathered per edge + neighbour ids
          + output rows + rowptr), divided by the mean step time.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E peak

# Bytes per launch that left the L2s for the default workload, from the hardware-counter runs
# summarised in profiles/propagate_copy_sum_1M_20M_F64.md (FETCH_SIZE x 2.000 calibration factor
# + WRITE_SIZE x 1.000).  Only meaningful for the default N/E/F; other sizes report null.
MEASURED_TRAFFIC_BYTES = {(1_000_000, 20_000_000, 64): int((1302746.4 * 2.0 + 254475.0) * 1024)}


def b_alg(n, e, f, weighted=False):
    return e * (4 * f + 4 + (4 if weighted else 0)) + n * 4 * f + (n + 1) * 4


def b_min(n, e, f, weighted=False):
    return 2 * n * 4 * f + e * (4 + (4 if weighted else 0)) + (n + 1) * 4


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


def cpu_baseline(wl, sample_edges):
    """The parity oracle as it stands (one thread, double accumulators) on a prefix of the edge list."""
    import oracle
    e = min(sample_edges, wl.num_edges)
    src, dst = wl.src[:e].copy(), wl.dst[:e].copy()
    t0 = time.perf_counter()
    oracle.propagate(src, dst, wl.num_nodes, wl.x)
    dt = time.perf_counter() - t0
    n, f = wl.x.shape
    return {"value": b_alg(n, e, f) / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"copy_xj+sum over the first {e} of {wl.num_edges} edges (all {n} nodes, F={f}), "
                      f"one pass, {dt:.1f} s", "seconds": dt, "edge_feature_per_s": e * f / dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--nodes", type=int, default=1_000_000)
    ap.add_argument("--edges", type=int, default=20_000_000)
    ap.add_argument("--feat", type=int, default=64)
    ap.add_argument("--cpu-sample-edges", type=int, default=10_000_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="time only the headline step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2412_06354_amd import binding as gnn, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    gnn.lib()
    torch.cuda.set_device(0)

    wl = synth.config2_weighted(num_nodes=args.nodes, num_edges=args.edges, feat=args.feat)
    n, e, f = wl.num_nodes, wl.num_edges, args.feat
    stats = wl.stats()
    src, dst = torch.from_numpy(wl.src).cuda(), torch.from_numpy(wl.dst).cuda()
    x = torch.from_numpy(wl.x).cuda()
    ew = torch.from_numpy(wl.edge_weight).cuda()
    out = torch.empty_like(x)

    t0 = time.perf_counter()
    g = gnn.build_csr(src, dst, n)
    torch.cuda.synchronize()
    build_first_ms = (time.perf_counter() - t0) * 1e3

    def step():
        gnn.propagate(g, x, None, gnn.MSG_COPY_XJ, gnn.AGGR_SUM, out=out)

    ms = time_calls(torch, step, args.steps, args.warmup)
    bytes_alg = b_alg(n, e, f)
    gbs = bytes_alg / (ms * 1e-3) / 1e9

    extra = {"graph": stats, "work_lists": g.work_sizes(), "B_alg_bytes": bytes_alg,
             "B_min_bytes": b_min(n, e, f), "t_min_over_t": b_min(n, e, f) / 8e12 / (ms * 1e-3),
             "edge_feature_per_s": e * f / (ms * 1e-3), "csr_build_first_call_ms": build_first_ms}
    # a plain streaming kernel (read 1 GiB, write 1 GiB) as a second denominator and as the
    # calibration dispatch for hardware-counter runs
    big = torch.zeros(256 * 1024 * 1024, dtype=torch.float32, device="cuda")
    big2 = torch.empty_like(big)
    copy_ms = time_calls(torch, lambda: torch.add(big, 1.0, out=big2), 10, 2)
    extra["copy_kernel_GBs"] = 2 * big.numel() * 4 / (copy_ms * 1e-3) / 1e9
    extra["copy_kernel_bytes_each_way"] = big.numel() * 4
    del big, big2
    if not args.no_extra:
        k = max(5, args.steps // 10)
        e_csr = gnn.edge_data_to_csr(g, ew)
        for name, msg, aggr in (("e_mul_xj_sum", 1, 0), ("e_mul_xj_mean", 1, 1), ("e_mul_xj_max", 1, 2),
                                ("copy_xj_mean", 0, 1), ("copy_xj_max", 0, 2)):
            ed = e_csr if msg else None
            t = time_calls(torch, lambda: gnn.propagate(g, x, ed, msg, aggr, e_order=gnn.EDGE_ORDER_CSR, out=out), k, 3)
            extra[name] = {"ms": t, "GBs_alg": b_alg(n, e, f, bool(msg)) / (t * 1e-3) / 1e9}
        t = time_calls(torch, lambda: gnn.propagate(g, x, ew, 1, 0, e_order=gnn.EDGE_ORDER_COO, out=out), k, 3)
        extra["e_mul_xj_sum_coo_order"] = {"ms": t, "GBs_alg": b_alg(n, e, f, True) / (t * 1e-3) / 1e9}
        t = time_calls(torch, lambda: gnn.edge_data_to_csr(g, ew), k, 2)
        extra["edge_data_to_csr_ms"] = t

        def rebuild():
            gnn.build_csr(src, dst, n).close()
        t0 = time.perf_counter()
        for _ in range(3):
            rebuild()
        torch.cuda.synchronize()
        extra["csr_build_ms"] = (time.perf_counter() - t0) / 3 * 1e3

    line = {
        "metric": "propagate(copy_xj,sum) algorithmic GB/s, 1M-node/20M-edge power-law graph, F=64",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "N": n, "E": e, "F": f, "msg": "copy_xj", "aggr": "sum",
                   "seed": synth.seed_of(2)},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get((n, e, f)),
                     "kernel": "propagate_kernel<16,4,copy_xj,sum> (+ combine_pieces_kernel, a few us)"},
        "extra": extra,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_edges)
    g.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
