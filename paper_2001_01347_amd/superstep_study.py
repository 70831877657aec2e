"""BSP against ElasticBSP on synthetic workers: waiting time over a run of supersteps.

    python -m paper_2001_01347_amd.superstep_study [--config 2] [--supersteps 64] [--sync-cost 2000]

The part of the paper's comparison (Section V-B: BSP against ElasticBSP with
R = 15, 30, 60, 120, 240 predicted iterations per worker) that needs only
iteration times: for every R the same synthetic workers run S supersteps through
``ebsp_simulate_supersteps`` (R = 1 is BSP with one iteration per superstep) and the
table shows where the workers' time went.  Every search runs in the HIP library;
this module only sums the per-superstep outputs (on the device) and prints them.
Accuracy and convergence, which the paper measures by training, are not modelled.
"""
from __future__ import annotations

import argparse
import sys
from typing import Dict, Iterable, List

PAPER_LOOKAHEADS = (15, 30, 60, 120, 240)       # the values of R in Section V-B


def summarise(last_end0, interval, sync_cost: int, barrier, iters, wait) -> Dict[str, float]:
    """Where the workers' time went in one run (tensors as ``ebsp_simulate_supersteps`` takes and returns them).

    Worker time counts from each worker's start to the last barrier.  It splits into computing
    (finished iterations), waiting at barriers and synchronising (``sync_cost`` after every barrier
    but the last); the three shares add up to 1.
    """
    S, B, P = (int(x) for x in interval.shape)
    total = float((barrier[S - 1][:, None] - last_end0).sum().item())
    waiting = float(wait.sum().item())
    syncing = float(sync_cost) * (S - 1) * B * P
    done = float(iters.sum().item())
    computing = float((iters.to(interval.dtype) * interval).sum().item())
    return {"supersteps": S, "iterations_per_superstep": done / (S * B * P),
            "wait_per_iteration": waiting / done, "waiting_share": waiting / total,
            "sync_share": syncing / total, "computing_share": computing / total,
            "iterations_per_worker_second": done / (total * 1e-6)}


def study(k: int = 2, lookaheads: Iterable[int] = (1,) + PAPER_LOOKAHEADS, supersteps: int = 64,
          instances: int = 256, sync_cost: int = 2000, jitter: float = 0.02) -> List[Dict[str, float]]:
    """One row per lookahead R for the workers of synthetic configuration ``k`` (times in microseconds)."""
    import torch
    from . import workloads, zipline

    n = min(int(instances), workloads.CONFIGS[k].B)
    le, iv = workloads.make_supersteps(k, supersteps, instances=range(n), jitter=jitter)
    le_dev, iv_dev = torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda()
    rows = []
    for R in lookaheads:
        barrier, iters, wait, status = zipline.ebsp_simulate_supersteps(le_dev, iv_dev, int(R), sync_cost)
        if int(status.max().item()) != 0:
            raise zipline.ZipLineError(f"R={R}: the search flagged an instance")
        row = {"R": int(R)}
        row.update(summarise(le_dev, iv_dev, sync_cost, barrier, iters, wait))
        rows.append(row)
    return rows


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4, 5], help="whose workers (2: 16 workers, 80-120 ms)")
    ap.add_argument("--supersteps", type=int, default=64)
    ap.add_argument("--instances", type=int, default=256, help="independent clusters averaged over")
    ap.add_argument("--sync-cost", type=int, default=2000, help="time from a barrier to the restart (us)")
    ap.add_argument("--jitter", type=float, default=0.02, help="relative spread of a worker's iteration time between supersteps")
    args = ap.parse_args()
    rows = study(args.config, (1,) + PAPER_LOOKAHEADS, args.supersteps, args.instances, args.sync_cost, args.jitter)
    print("| R | iterations per superstep and worker | wait per iteration (us) | waiting | synchronising | computing | iterations per worker-second |")
    print("|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['R']}{' (BSP)' if r['R'] == 1 else ''} | {r['iterations_per_superstep']:.2f} | {r['wait_per_iteration']:.0f} | "
              f"{100 * r['waiting_share']:.2f} % | {100 * r['sync_share']:.2f} % | {100 * r['computing_share']:.2f} % | "
              f"{r['iterations_per_worker_second']:.3f} |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
