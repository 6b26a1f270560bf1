#!/usr/bin/env python3
"""Benchmark: batched NotebookOS policy replays on one MI355X.

A "step" is one pass of the whole hot path (placement, election, commit/release, migration,
scale-out/in, queueing, final drain) over one batch of synthetic traces that is already resident
in HBM. Metric: cell events x initial hosts per second, summed over the replays of the batch.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--replays N]
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

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published


def measured_traffic(workload: str):
    """HBM bytes per launch from the committed rocprofv3 counter runs (profiles/hbm_traffic.json),
    or None when the kernel sources have changed since they were taken."""
    import glob
    import hashlib
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json"))).get(workload)
    except OSError:
        return None
    if not rec:
        return None
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2503_20591_amd", "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return rec["traffic_bytes"] if h.hexdigest() == rec["csrc_sha256"] else None


def cpu_baseline(batch, budget_s: float, threads: int):
    """The CPU oracle, as it stands, timed on a bounded sample of the same batch."""
    import oracle
    oracle.build()
    per_cells = batch.n_cells() / max(batch.n_replays, 1)
    # one replay first to size the sample
    t0 = time.perf_counter()
    oracle.replay_batch(batch, replays=[0])
    one = max(time.perf_counter() - t0, 1e-6)
    n = int(max(1, min(batch.n_replays, budget_s * threads / one)))
    idx = [int(i * batch.n_replays / n) for i in range(n)]
    t0 = time.perf_counter()
    oracle.replay_batch(batch, replays=idx, threads=threads)
    dt = time.perf_counter() - t0
    value = per_cells * n * batch.config["hosts_initial"] / dt
    return {"value": value, "unit": "cell-events*hosts/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {batch.n_replays} replays of {batch.name}, evenly spaced, "
                      f"{threads} thread(s), {dt:.1f} s"}


def measured_copy_gbs(torch):
    """What a plain device-to-device copy reaches on this GPU (bytes read + written per second): the
    achievable HBM rate the 8 TB/s vendor peak is put beside."""
    n = 512 * 1024 * 1024
    src = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "c4a", "c2b", "c4b", "c2l", "c4l"])
    ap.add_argument("--replays", type=int, default=None, help="truncate the batch (for quick looks)")
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time; 0 = skip")
    ap.add_argument("--cpu-threads", type=int, default=0, help="0 = all host cores (at most 16)")
    ap.add_argument("--hosts-in-lds", action="store_true", help="force the any-size kernel (comparison runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (replays are independent; a multi-GPU run "
              "would only split the batch). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_20591_amd import replay, tracegen
    replay.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    t0 = time.perf_counter()
    batch = tracegen.workload(args.workload, n_replays=args.replays, workers=min(16, os.cpu_count() or 1))
    t_gen = time.perf_counter() - t0
    t0 = time.perf_counter()
    dev = replay.upload(batch, "cuda:0")
    torch.cuda.synchronize()
    t_up = time.perf_counter() - t0
    if args.calibrate_copy:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    h = replay.Replay(batch.config, dev, hosts_in_lds=args.hosts_in_lds)
    info = h.launch_info()

    for _ in range(args.warmup):
        h.run()
    torch.cuda.synchronize()
    kernel_ms = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        h.run()
        kernel_ms.append(None)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # per-launch device time from the library's HIP events on its own stream (one extra timed pass
    # per sample, outside the wall-clock region above)
    dur = []
    for _ in range(min(args.steps, 10)):
        h.run()
        dur.append(h.last_kernel_ms())
    st = h.stats()
    assert (st["status"] == 0).all()
    h.close()
    copy_gbs = measured_copy_gbs(torch)

    ms_per_step = wall * 1e3 / args.steps
    cells = batch.n_cells()
    value = cells * batch.config["hosts_initial"] / (ms_per_step * 1e-3)
    alg_bytes = batch.algorithmic_bytes(replay.STATS_DTYPE.itemsize)
    avg_kernel_ms = sum(dur) / len(dur)
    achieved = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9

    threads = args.cpu_threads or min(16, os.cpu_count() or 1)
    cpu = cpu_baseline(batch, args.cpu_budget, threads) if args.cpu_budget > 0 else None

    out = {
        "metric": "replayed cell events x hosts scored / sec on 1 MI355X",
        "value": value, "unit": "cell-events*hosts/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{batch.name}: {batch.n_replays} replays x {batch.config['hosts_initial']} hosts "
                               f"(max {batch.config['hosts_max']}) x {batch.config['gpus_per_host']} GPUs, "
                               f"{cells // max(batch.n_replays, 1)} cell events/replay",
                   "replays": batch.n_replays, "events_total": batch.n_events(), "cell_events_total": cells,
                   "events_per_s": batch.n_events() / (ms_per_step * 1e-3),
                   "lds_bytes_per_replay": info["lds_bytes"], "threads_per_group": info["threads_per_group"],
                   "gen_s": round(t_gen, 2), "upload_s": round(t_up, 2)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "copy_gbs": copy_gbs, "frac_of_copy": achieved / copy_gbs,
                     "traffic": None if (args.replays or args.hosts_in_lds) else measured_traffic(args.workload),
                     "kernel": "nbos_replay_kernel", "kernel_ms": avg_kernel_ms, "algorithmic_bytes": alg_bytes,
                     "ns_per_event_per_replay": avg_kernel_ms * 1e6 / (batch.n_events() / max(batch.n_replays, 1))},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
