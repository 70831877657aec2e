#!/usr/bin/env python3
"""Benchmark of the batched ZipLine barrier search on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5]

A step is one ``ebsp_zipline_batch`` call (every kernel of the search) over
one synthetic batch that is already resident in HBM.  The default workload is
the largest configuration (B=64 instances, P=1024 workers, R=4096 lookahead,
268 435 456 int64 timestamps, 2 GiB).  Prints ONE JSON line with the
throughput in timestamps/s (and instances/s), the roofline figures of the
kernel that takes the most time (measured live with HIP events recorded around
every kernel launch on the stream the kernels run on), and the CPU oracle
timed on the host cores over a bounded sample of the same workload.
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
# reads for the plain copy kernel of known size (FETCH_SIZE x 2048 B, WRITE_SIZE x 1024 B per count).  They
# hold only for the kernel sources they were taken from: `traffic` is null once those have changed.
COUNTED_SOURCES_SHA256 = "f835e57ff9849d4afdfdffc2214efd5caabfed39a751a349f7489bac15061102"
COUNTED_TRAFFIC = {     # (objective, predicted, config) -> (dominant kernel, its bytes, bytes of all kernels of a call)
    ("sum", False, 5): ("zl_window_kernel", 2260923 * 2048 + 1223 * 1024, 7542405397),
    ("sum", False, 3): ("zl_instance_kernel", 1189601 * 2048 + 5655 * 1024, 2459061408),
    ("range", False, 5): ("zl_range_fast_kernel", 2233769 * 2048 + 1684 * 1024, 7495621707),
    ("sum", True, 5): ("zl_window_kernel", 267418 * 2048 + 562 * 1024, 1176893707),
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
    if kernel == "zl_instance_kernel":      # every timestamp once, all three outputs
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
    if kernel == "zl_finish_kernel":        # window results; per row its crossing indices at the barrier's bin and two probes
        import math                         # (predicted rows: nothing is probed), outputs
        probes = 0.0 if predicted else 64.0 * 3.0
        return 16.0 * windows + B * P * (probes + 4.0) + 16.0 * B
    return 0.0


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
    ap.add_argument("--window-cap", type=int, default=0, help="tuning: records per window workgroup (0: default)")
    ap.add_argument("--window-fill", type=int, default=0, help="tuning: entries a window is filled to (0: default)")
    ap.add_argument("--single-max", type=int, default=0, help="tuning: largest P*R taken by one workgroup (0: default)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on exactly one GPU (instances are independent and would "
              "shard over B with no exchange, but no multi-GPU path is part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2001_01347_amd import workloads, zipline

    zipline.ebsp_zipline_tune(args.window_cap, args.single_max, args.window_fill)
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

    # timed region: K steps, per-kernel HIP events recorded inside the library on the launch stream
    searches = max(1, S)                    # searches (launches of every kernel of the search) per step
    n_keys *= searches                      # timestamps a step looks through
    zipline.ebsp_zipline_profile_begin(args.steps * searches)
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    w1 = time.perf_counter()
    kernel_ms, calls = zipline.ebsp_zipline_profile_end()
    assert calls == args.steps * searches
    ms_per_step = (w1 - w0) * 1e3 / args.steps
    assert int(status.max().item()) == 0, "the search flagged a data error on synthetic input"

    # yardstick: a plain streaming copy of the same 8 B/key input (reads and writes n_keys * 8 bytes)
    copy_gbs = None
    if args.copy_probe > 0 and ts is not None:
        dst = torch.empty_like(ts)
        zipline.ebsp_zipline_copy_probe(ts, dst)
        torch.cuda.synchronize()
        zipline.ebsp_zipline_profile_begin(args.copy_probe)
        for _ in range(args.copy_probe):
            zipline.ebsp_zipline_copy_probe(ts, dst)
        copy_ms, ncopy = zipline.ebsp_zipline_profile_end()
        copy_gbs = 2.0 * 8.0 * n_keys / (copy_ms["zl_copy_kernel"] / ncopy * 1e-3) / 1e9
        del dst

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
    dom = max(per_kernel, key=per_kernel.get)
    dom_bytes = algorithmic_bytes(dom, B, P, R, bins, windows, args.predicted)
    achieved = dom_bytes / (per_kernel[dom] * 1e-3) / 1e9
    counted = COUNTED_TRAFFIC.get((args.objective, bool(args.predicted), args.config))
    tuned = bool(args.window_cap or args.single_max or args.window_fill)
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
    n_one = max(1, n_cpu // cores)                          # the same oracle on one thread, a sixteenth of the sample
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
                         "matches_gpu": bool(same), "one_thread_value": cpu_rate_one, "cpu_model": cpu_model},
        "copy_probe_GBs": copy_gbs,
        "setup_s": gen_s,
    }
    print(json.dumps(out))
    if not same:
        print("bench.py: the GPU results differ from the CPU oracle on the sampled instances", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
