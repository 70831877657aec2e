#!/usr/bin/env python3
"""Benchmark of the batched ZipLine barrier search on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5]

A step is one ``ebsp_zipline_batch`` call (every kernel of the search) over
one synthetic batch that is already resident in HBM.  The default workload is
the largest configuration (B=64 instances, P=1024 workers, R=4096 lookahead,
268 435 456 int64 timestamps, 2 GiB).  Prints ONE JSON line with the
throughput in timestamps/s (and instances/s), the roofline figures of the
kernel that takes the most time, and the CPU oracle timed on the host cores
over a bounded sample of the same workload.

Two passes over the same K steps: the first is the headline (wall clock around
all K calls, plus one HIP event pair around every call on the launch stream:
median and mean), with nothing recorded inside the library; the second repeats
the K calls with a HIP event pair around every kernel launch and gives the
per-kernel durations that the roofline figures use.

``--table2`` runs the shapes of the paper's Table II instead (10, 100, 1000
workers; 15 and 150 predicted iterations): ZipLine against GridScan and
FullGridScan, their run times and how far the heuristics' d_Z is from the
optimum.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


# HBM bytes per launch of the dominant kernel, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of
# this program (their summaries, with the commands, are under profiles/), each scaled by what the same counter
# reads for the plain copy kernel of known size (FETCH_SIZE x 2048 B, WRITE_SIZE x 1024 B per count).  The
# figures below are the counters' per-dispatch averages, kernel by kernel in launch order.  They hold only for
# the kernel sources they were taken from: `traffic` is null once those have changed.
COUNTED_SOURCES_SHA256 = "8a357e189d87dc08d46985853e941fb98f575fecc7a2489b26f751e3dec9a5a9"
FETCH_UNIT, WRITE_UNIT = 2048, 1024      # bytes per count: what the copy kernel's 2 GiB in, 2 GiB out read as (1 048 607 and 2 097 152)
COUNTED_TRAFFIC = {     # (objective, predicted, config) -> (dominant kernel, its bytes, bytes of all kernels of a call)
    ("sum", False, 5): ("zl_window_kernel", 2263792 * FETCH_UNIT + 1238 * WRITE_UNIT,
                        (16448 + 1049297 + 35886 + 658 + 2263792 + 358 + 8502) * FETCH_UNIT
                        + (70 + 608424 + 1025 + 1239 + 1238 + 8192 + 258) * WRITE_UNIT),
    ("sum", False, 3): ("zl_instance_reg_kernel", 1405244 * FETCH_UNIT + 144188 * WRITE_UNIT,
                        (1405244 + 97) * FETCH_UNIT + (144188 + 16384) * WRITE_UNIT),
    ("range", False, 5): ("zl_range_fast_kernel", 2461671 * FETCH_UNIT + 2071 * WRITE_UNIT,
                          (16447 + 1049295 + 35886 + 670 + 2461671 + 617 + 8911) * FETCH_UNIT
                          + (70 + 608466 + 1025 + 1716 + 2071 + 14459 + 258) * WRITE_UNIT),
    ("sum", True, 5): ("zl_window_kernel", 267414 * FETCH_UNIT + 561 * WRITE_UNIT,
                       (575 + 10356 + 9004 + 658 + 267414 + 357 + 1666) * FETCH_UNIT
                       + (582 + 548866 + 1024 + 1240 + 561 + 8192 + 258) * WRITE_UNIT),
    ("sum", False, 4): ("zl_window_kernel", 2054930 * FETCH_UNIT + 2672 * WRITE_UNIT,
                        (65606 + 1053106 + 18132 + 1875 + 2054930 + 656 + 36371) * FETCH_UNIT
                        + (1120 + 306295 + 2048 + 2519 + 2672 + 0 + 1088) * WRITE_UNIT),
}


def kernel_sources_sha256() -> str:
    """Hash of the HIP sources the library is built from (file names and contents, in name order)."""
    import hashlib
    d = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2001_01347_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def algorithmic_bytes(kernel: str, B: int, P: int, R: int, bins: int, windows: int, predicted: bool = False) -> float:
    """Bytes a kernel must move per launch (inputs it has to read once + what it has to write)."""
    n = float(B) * P * R
    cw = 2.0 if R < 65536 else 4.0          # bytes of one crossing index
    rows = 16.0 * B * P if predicted else 8.0 * n       # predicted rows: 16 bytes per worker stand for R timestamps
    if kernel in ("zl_instance_kernel", "zl_instance_reg_kernel"):      # every timestamp once, all three outputs
        return rows + B * (16.0 + 4.0 * P)
    if kernel == "zl_window_kernel":        # every timestamp once, two crossing rows per window, one result
        return rows + windows * (2.0 * cw * P + 16.0)
    groups = (P + 63) // 64 if predicted else (P + 15) // 16    # rows of partial column sums per instance (stored rows: when the bins fit LDS)
    if kernel == "zl_partition_kernel":     # every timestamp once, one crossing index per (row, bin), partial column sums
        return 8.0 * n + cw * B * P * (bins + 1) + (4.0 * B * groups * (bins + 1) if bins + 1 <= 8200 else 0.0)
    if kernel == "zl_partition_pred_kernel":    # 16 bytes per worker, one crossing index per (row, bin), partial column sums
        return 16.0 * B * P + cw * B * P * (bins + 1) + 4.0 * B * ((P + 63) // 64) * (bins + 1)
    if kernel == "zl_bincount_kernel":      # the partial column sums once (else the crossing indices), one count per bin
        return (4.0 * B * groups if predicted or bins + 1 <= 8200 else cw * B * P) * (bins + 1) + 4.0 * B * (bins + 1)
    if kernel == "zl_bounds_kernel":        # first and last timestamp of every row (one 64-byte line each)
        return 128.0 * B * P
    if kernel == "zl_plan_kernel":
        return 4.0 * B * (bins + 1) + 4.0 * windows
    if kernel in ("zl_range_fast_kernel", "zl_range_window_kernel"):
        # every timestamp once (a neighbour comes in the same line), crossing rows, one result.  The sort-based
        # kernel only takes the windows the fast one leaves to it: priced at the whole input, its figure is a ceiling.
        return 8.0 * n + windows * (2.0 * cw * P + 16.0)
    if kernel == "zl_range_instance_kernel":
        return 8.0 * n + B * (16.0 + 4.0 * P)
    if kernel == "zl_sweep_kernel":         # every timestamp once, one partial result per slice
        return rows + 16.0 * windows
    if kernel == "zl_sweep_finish_kernel":  # partial results; per row two probes of its entries, outputs
        return 16.0 * windows + B * P * (64.0 * 2.0 + 4.0) + 16.0 * B
    if kernel == "zl_finish_kernel":        # window results; per row its crossing indices at the barrier's bin and two probes
        import math                         # (predicted rows: nothing is probed), outputs
        probes = 0.0 if predicted else 64.0 * 3.0
        return 16.0 * windows + B * P * (probes + 4.0) + 16.0 * B
    return 0.0


# Table II of the paper (run time in microseconds on its 24-core Xeon server, mean of 10 trials): context only.
PAPER_TABLE2_US = {   # (workers, R) -> (ZipLine, FullGridScan, GridScan)
    (10, 15): (1.49e2, 1.54e3, 1.68e2), (10, 150): (1.32e3, 4.67e4, 5.50e3),
    (100, 15): (6.37e3, 8.13e4, 1.11e3), (100, 150): (4.99e4, 2.15e6, 4.38e4),
    (1000, 15): (2.53e5, 4.04e6, 7.45e3), (1000, 150): (2.38e6, 2.07e8, 2.57e5),
}


def table2(args) -> int:
    """The comparison of Section V-A (Table II) on synthetic workers: per shape, a batch of instances searched by
    ZipLine (the paper's objective max(Z) - min(Z), and the summed wait), GridScan and FullGridScan on the GPU."""
    import numpy as np
    import torch
    import oracle
    from paper_2001_01347_amd import workloads, zipline

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    rows, ok = [], True
    n_inst = max(1, args.table2_instances)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ms = []
        for _ in range(max(10, args.steps)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ms.append(e0.elapsed_time(e1))
        return float(np.median(ms)), float(np.mean(ms))

    for P in (10, 100, 1000):
        for R in (15, 150):
            host = workloads.make_workers(P, R, n_inst)
            ts = torch.from_numpy(host).to(dev)
            res, times = {}, {}
            for name, fn in (("zipline_range", lambda: zipline.ebsp_zipline_range_batch(ts)),
                             ("zipline_sum", lambda: zipline.ebsp_zipline_batch(ts)),
                             ("gridscan", lambda: zipline.ebsp_gridscan_batch(ts, False)),
                             ("fullgridscan", lambda: zipline.ebsp_gridscan_batch(ts, True))):
                out = fn()
                torch.cuda.synchronize()
                assert int(out[3].max().item()) == 0
                res[name] = [t.cpu().numpy() for t in out[:3]]
                times[name] = timed(fn)
            opt, gs, fgs = res["zipline_range"][2], res["gridscan"][2], res["fullgridscan"][2]
            # the oracle on a bounded sample (FullGridScan costs P^2 R log R per instance on the CPU)
            n_cpu = max(1, min(n_inst, int(2e9 // (P * P * R * 8)) or 1))
            c0 = time.perf_counter()
            o_gs = oracle.gridscan(host[:n_cpu], False, "bisect")
            o_fgs = oracle.gridscan(host[:n_cpu], True, "bisect")
            o_opt = oracle.zipline_range(host[:n_cpu])
            cpu_s = time.perf_counter() - c0
            same = all(np.array_equal(a[i][:n_cpu], o[i]) for a, o in ((res["gridscan"], o_gs), (res["fullgridscan"], o_fgs),
                                                                       (res["zipline_range"], o_opt)) for i in range(3))
            ok &= bool(same) and bool((fgs <= gs).all()) and bool((opt <= fgs).all())
            paper = PAPER_TABLE2_US[(P, R)]
            rows.append({
                "workers": P, "R": R, "instances": n_inst,
                "us_per_instance": {k: v[0] * 1e3 / n_inst for k, v in times.items()},
                "batch_ms_median": {k: v[0] for k, v in times.items()},
                "batch_ms_mean": {k: v[1] for k, v in times.items()},
                "d_Z_mean": {"zipline": float(opt.mean()), "gridscan": float(gs.mean()), "fullgridscan": float(fgs.mean())},
                "d_Z_over_optimum_mean": {"gridscan": float((gs / np.maximum(opt, 1)).mean()),
                                          "fullgridscan": float((fgs / np.maximum(opt, 1)).mean())},
                "finds_optimum_frac": {"gridscan": float((gs == opt).mean()), "fullgridscan": float((fgs == opt).mean())},
                "oracle": {"instances": n_cpu, "matches_gpu": bool(same), "seconds": cpu_s},
                "paper_us_xeon": {"zipline": paper[0], "fullgridscan": paper[1], "gridscan": paper[2]},
            })
    print(json.dumps({"metric": "table2_search_time", "unit": "us/instance", "n_gpus": 1, "dtype": "int64", "data": "synthetic",
                      "config": {"workload": f"Table II shapes, {n_inst} instances per shape in one batch, "
                                             "workers with mean iteration time U[80,120] ms, LogNormal(0, 0.1) jitter"},
                      "rows": rows}))
    if not ok:
        print("bench.py: a GPU result differs from the CPU oracle, or the heuristics beat the optimum", file=sys.stderr)
        return 1
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--objective", default="sum", choices=["sum", "range"],
                    help="sum: the summed waiting time (ebsp_zipline_batch, the default); "
                         "range: the paper's formal objective max(Z) - min(Z) (ebsp_zipline_range_batch)")
    ap.add_argument("--predicted", action="store_true",
                    help="rows predicted inside the kernels from (last_end, interval) per worker "
                         "(ebsp_predict_zipline_batch): nothing but 16 bytes per worker is read from HBM")
    ap.add_argument("--supersteps", type=int, default=0,
                    help="S > 0: a step is one ebsp_simulate_supersteps call, S supersteps of predict -> search -> "
                         "resume at the barrier on the device (implies --predicted)")
    ap.add_argument("--sync-cost", type=int, default=2000, help="with --supersteps: time from a barrier to the restart (us)")
    ap.add_argument("--cpu-instances", type=int, default=-1,
                    help="instances in the CPU-oracle sample (default: sized for roughly 10-30 s of CPU work)")
    ap.add_argument("--copy-probe", type=int, default=3,
                    help="launches of the plain copy kernel (the input's size) after the timed region; "
                         "its bandwidth and byte counters are the yardstick for the others (0: skip)")
    ap.add_argument("--table2", action="store_true",
                    help="the shapes of the paper's Table II instead: ZipLine, GridScan and FullGridScan, times and d_Z")
    ap.add_argument("--table2-instances", type=int, default=64, help="with --table2: instances per shape")
    ap.add_argument("--sweep-min", type=int, default=0,
                    help="tuning: smallest P*R searched by the frontier sweep (0: default, negative: never)")
    ap.add_argument("--slice-keys", type=int, default=0, help="tuning: entries per slice of the frontier sweep (0: default)")
    ap.add_argument("--sweep-lines", type=int, default=0, help="tuning: 128-byte lines a window of the frontier sweep asks for (0: default)")
    ap.add_argument("--window-cap", type=int, default=0, help="tuning: records per window workgroup (0: default)")
    ap.add_argument("--window-fill", type=int, default=0, help="tuning: entries a window is filled to (0: default)")
    ap.add_argument("--single-max", type=int, default=0, help="tuning: largest P*R taken by one workgroup (0: default)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on exactly one GPU (instances are independent and would "
              "shard over B with no exchange, but no multi-GPU path is part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be at least 1 and --warmup at least 0", file=sys.stderr)
        return 2
    if args.table2:
        return table2(args)

    import numpy as np
    import torch
    from paper_2001_01347_amd import workloads, zipline

    zipline.ebsp_zipline_tune(args.window_cap, args.single_max, args.window_fill)
    zipline.ebsp_zipline_tune_sweep(args.sweep_min, args.slice_keys, args.sweep_lines)
    cfg = workloads.CONFIGS[args.config]
    B, P, R = cfg.B, cfg.P, cfg.R
    n_keys = cfg.n_keys
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    S = max(0, args.supersteps)
    if S:
        args.predicted = True
    t0 = time.time()
    if S:
        if args.objective != "sum":
            print("bench.py: --supersteps goes with the summed-wait objective only", file=sys.stderr)
            return 2
        le_host, iv_host = workloads.make_supersteps(args.config, S)
        le_dev, iv_dev = torch.from_numpy(le_host).to(dev), torch.from_numpy(iv_host).to(dev)
        host = ts = None
    elif args.predicted:
        if args.objective != "sum":
            print("bench.py: --predicted goes with the summed-wait objective only", file=sys.stderr)
            return 2
        le_host, iv_host = workloads.make_predicted(args.config)
        le_dev, iv_dev = torch.from_numpy(le_host).to(dev), torch.from_numpy(iv_host).to(dev)
        host = ts = None
    else:
        host = workloads.make(args.config, threads=16)
        ts = torch.from_numpy(host).to(dev)
    gen_s = time.time() - t0

    lead = (S,) if S else ()
    barrier = torch.empty(lead + (B,), dtype=torch.int64, device=dev)
    iters = torch.empty(lead + (B, P), dtype=torch.int32, device=dev)
    wait = torch.empty(lead + (B,), dtype=torch.int64, device=dev)
    status = torch.empty(lead + (B,), dtype=torch.int32, device=dev)
    ranged = args.objective == "range"
    ws_bytes = (zipline.ebsp_simulate_workspace_bytes if S else zipline.ebsp_zipline_range_workspace_bytes if ranged
                else zipline.ebsp_predict_zipline_workspace_bytes if args.predicted
                else zipline.ebsp_zipline_workspace_bytes)(B, P, R)
    workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def step():
        if S:
            zipline.ebsp_simulate_supersteps(le_dev, iv_dev, R, args.sync_cost, barrier, iters, wait, status, workspace)
        elif args.predicted:
            zipline.ebsp_predict_zipline_batch(le_dev, iv_dev, R, barrier, iters, wait, status, workspace)
        elif ranged:
            zipline.ebsp_zipline_range_batch(ts, barrier, iters, wait, status, workspace)
        else:
            zipline.ebsp_zipline_batch(ts, barrier, iters, wait, status, workspace)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # pass 1, the headline: K steps with nothing recorded inside the library.  Wall clock around all of them
    # (ms_per_step) and one HIP event pair per call on the launch stream (torch's current stream, the one the
    # binding hands to the library): median and mean.
    searches = max(1, S)                    # searches (launches of every kernel of the search) per step
    n_keys *= searches                      # timestamps a step looks through
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for e0, e1 in ev:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    w1 = time.perf_counter()
    ms_per_step = (w1 - w0) * 1e3 / args.steps
    call_ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    call_ms_median = call_ms[len(call_ms) // 2] if len(call_ms) % 2 else 0.5 * (call_ms[len(call_ms) // 2 - 1] + call_ms[len(call_ms) // 2])
    call_ms_mean = sum(call_ms) / len(call_ms)
    assert int(status.max().item()) == 0, "the search flagged a data error on synthetic input"

    # pass 2: the same K steps with a HIP event pair around every kernel launch (recorded inside the library on
    # the launch stream): per-kernel durations for the roofline figures
    zipline.ebsp_zipline_profile_begin(args.steps * searches)
    for _ in range(args.steps):
        step()
    kernel_ms, calls = zipline.ebsp_zipline_profile_end()
    assert calls == args.steps * searches

    # yardsticks over the same 8 B/key input: a plain streaming copy (reads and writes n bytes) and a plain
    # streaming read; and the peak that the device's own memory clock and bus width imply
    copy_gbs = read_gbs = None
    if args.copy_probe > 0 and ts is not None:
        nbytes = ts.numel() * 8
        dst = torch.empty_like(ts)
        sink = torch.zeros(zipline.READ_SINK_WORDS, dtype=torch.int64, device=dev)
        zipline.ebsp_zipline_copy_probe(ts, dst)
        zipline.ebsp_zipline_read_probe(ts, sink)
        torch.cuda.synchronize()
        zipline.ebsp_zipline_profile_begin(2 * args.copy_probe)
        for _ in range(args.copy_probe):
            zipline.ebsp_zipline_copy_probe(ts, dst)
        for _ in range(args.copy_probe):
            zipline.ebsp_zipline_read_probe(ts, sink)
        probe_ms, nprobe = zipline.ebsp_zipline_profile_end()
        copy_gbs = 2.0 * nbytes / (probe_ms["zl_copy_kernel"] / args.copy_probe * 1e-3) / 1e9
        read_gbs = 1.0 * nbytes / (probe_ms["zl_read_kernel"] / args.copy_probe * 1e-3) / 1e9
        del dst
    mem_khz, mem_bits = zipline.ebsp_zipline_memory_info()
    device_peak_gbs = 2.0 * mem_khz * 1e3 * mem_bits / 8.0 / 1e9       # double data rate

    # shape-dependent constants of the multi-window path (for the byte model only)
    shape = zipline.ebsp_zipline_shape_info(B, P, R)
    bins = shape["bins"]
    if ranged and P * R > 8192 and not shape["multi"]:
        # this objective cuts instances of more than 8192 entries into windows: the shape as the library plans it
        zipline.ebsp_zipline_tune(args.window_cap, 8192, args.window_fill)
        shape = zipline.ebsp_zipline_shape_info(B, P, R)
        zipline.ebsp_zipline_tune(args.window_cap, args.single_max, args.window_fill)
    fill = shape["window_fill"]
    if ranged and shape["multi"]:           # this objective leaves room for its short list behind a window's entries
        fill -= shape["window_cap"] // (2 if P < 128 else 4)
    windows = B * ((P * R + fill - 1) // fill) if shape["multi"] else 0
    per_kernel = {k: v / calls for k, v in kernel_ms.items() if v > 0.0}      # per launch
    if "zl_sweep_kernel" in per_kernel:     # the frontier sweep: one partial result per slice, no windows
        windows = B * shape["slices"]
    dom = max(per_kernel, key=per_kernel.get)
    dom_bytes = algorithmic_bytes(dom, B, P, R, bins, windows, args.predicted)
    achieved = dom_bytes / (per_kernel[dom] * 1e-3) / 1e9
    counted = COUNTED_TRAFFIC.get((args.objective, bool(args.predicted), args.config))
    tuned = bool(args.window_cap or args.single_max or args.window_fill or args.sweep_min or args.slice_keys or args.sweep_lines)
    traffic = call_traffic = None
    if counted and counted[0] == dom and not tuned and not S and kernel_sources_sha256() == COUNTED_SOURCES_SHA256:
        traffic, call_traffic = float(counted[1]), float(counted[2])
    total_bytes = searches * sum(algorithmic_bytes(k, B, P, R, bins, windows, args.predicted) for k in per_kernel)

    # CPU oracle on a bounded sample of the same workload (baseline, not a target)
    import oracle
    cores = os.cpu_count() or 1
    cores = min(cores, 16)
    if args.cpu_instances > 0:
        n_cpu = min(B, args.cpu_instances)
    else:
        n_cpu = max(1, min(B, int(1.7e7 * cores // (P * R * searches)) or 1))
    # the same oracle on one thread: the first min(B, 64) instances, fewer where those would take over ~20 s
    n_one = max(1, min(B, 64, int(3.0e8 // (P * R * searches)) or 1))
    if S:
        oracle.simulate(le_host[:1], iv_host[:1, :1], R, args.sync_cost, threads=1)     # load the library
        c0 = time.perf_counter()
        ob, oi, ow, rc, used = oracle.simulate(le_host[:n_cpu], iv_host[:, :n_cpu], R, args.sync_cost, threads=cores)
        c1 = time.perf_counter()
        c2 = time.perf_counter()
        oracle.simulate(le_host[:n_one], iv_host[:, :n_one], R, args.sync_cost, threads=1)
        one_s = time.perf_counter() - c2
    else:
        sample = host[:n_cpu] if host is not None else oracle.predicted_rows(le_host[:n_cpu], iv_host[:n_cpu], R)
        cpu_search = oracle.zipline_range if ranged else oracle.zipline
        cpu_search(sample[:1], "sweep", threads=1)          # load the library, touch the pages
        c0 = time.perf_counter()
        ob, oi, ow, rc, used = cpu_search(sample, "sweep", threads=cores)
        c1 = time.perf_counter()
        c2 = time.perf_counter()
        cpu_search(sample[:n_one], "sweep", threads=1)
        one_s = time.perf_counter() - c2
    cpu_rate = n_cpu * P * R * searches / (c1 - c0)
    cpu_rate_one = n_one * P * R * searches / one_s
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
    except OSError:
        pass
    same = (np.array_equal(ob, barrier[..., :n_cpu].cpu().numpy())
            and np.array_equal(ow, wait[..., :n_cpu].cpu().numpy())
            and np.array_equal(oi, (iters[:, :n_cpu] if S else iters[:n_cpu]).cpu().numpy()))

    out = {
        "metric": ("elasticbsp_simulated_timestamps_per_sec" if S else
                   "zipline_predicted_timestamps_per_sec" if args.predicted else
                   "zipline_timestamps_per_sec" if not ranged else "zipline_range_timestamps_per_sec"),
        "value": n_keys / (ms_per_step * 1e-3),
        "unit": "timestamps/s",
        "instances_per_sec": B / (ms_per_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "call_ms_median": call_ms_median,
        "call_ms_mean": call_ms_mean,
        "call_ms_min": call_ms[0],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int64",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.k}: B={B} instances, P={P} workers, R={R} lookahead, "
                               f"{n_keys} int64 us timestamps " +
                               (f"predicted on the device over {S} supersteps" if S else "resident in HBM"),
                   "B": B, "P": P, "R": R, "objective": args.objective, "predicted": bool(args.predicted),
                   "supersteps": S},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel_ms": per_kernel[dom], "algorithmic_bytes": dom_bytes},
        "whole_call": {"algorithmic_bytes": total_bytes,
                       "achieved_GBs": total_bytes / (ms_per_step * 1e-3) / 1e9,
                       "floor_bytes": 8.0 * n_keys,
                       "floor_GBs": 8.0 * n_keys / (ms_per_step * 1e-3) / 1e9,
                       # HBM bytes the counters saw over all kernels of a call (null under the same conditions as
                       # roofline.traffic) against the call's duration: the traffic-based fraction of the HBM peak
                       "counted_bytes": call_traffic,
                       "counted_GBs": call_traffic / (ms_per_step * 1e-3) / 1e9 if call_traffic else None,
                       "counted_frac_of_peak": call_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS if call_traffic else None,
                       "kernel_ms": per_kernel},
        "cpu_baseline": {"value": cpu_rate, "unit": "timestamps/s", "cores": used, "kind": "oracle",
                         "sample": f"sweep oracle on the first {n_cpu} of {B} instances "
                                   f"({n_cpu * P * R * searches} timestamps), {c1 - c0:.2f} s wall",
                         "matches_gpu": bool(same), "one_thread_value": cpu_rate_one,
                         "one_thread_sample": f"the first {n_one} instances, {one_s:.2f} s", "cpu_model": cpu_model},
        "copy_probe_GBs": copy_gbs,
        "read_probe_GBs": read_gbs,
        "device_memory": {"clock_khz": mem_khz, "bus_bits": mem_bits, "implied_peak_GBs": device_peak_gbs},
        "setup_s": gen_s,
    }
    print(json.dumps(out))
    if not same:
        print("bench.py: the GPU results differ from the CPU oracle on the sampled instances", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
