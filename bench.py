#!/usr/bin/env python3
"""Benchmark: batched NotebookOS policy replays on one MI355X.

A "step" is one pass of the whole hot path (placement, election, commit/release, migration,
scale-out/in, queueing, final drain) over one batch of synthetic traces that is already resident
in HBM. Metric: cell events x initial hosts per second, summed over the replays of the batch.
The default workload is the largest one (c4: 256 replays of 512 -> 768 hosts, 8,000 sessions and
500,000 cells each). Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--replays N]
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
GPU_BOX_CPU_SHARE = 16    # host threads one GPU's share of the box allows


COMPUTE_UNITS = 256       # MI355X
CLOCK_HZ = 2.4e9


def counter_record(workload: str):
    """What the committed rocprofv3 counter runs read for one launch of this workload
    (profiles/hbm_traffic.json), or None when the kernel sources have changed since they were taken."""
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
    return rec if h.hexdigest() == rec["csrc_sha256"] else None


def measured_traffic(workload: str):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size), or None."""
    rec = counter_record(workload)
    return rec["traffic_bytes"] if rec else None


def issue_rates(workload: str, kernel_s: float):
    """Instructions the launch executes (counter runs) over the launch time measured here, per clock and
    compute unit. A compute unit issues at most one scalar and one vector wave-instruction per clock
    (one scalar unit; four SIMDs that take a wave64 vector instruction every four clocks)."""
    rec = counter_record(workload)
    if not rec or "insts_salu" not in rec:
        return None
    per = lambda n: n / (kernel_s * COMPUTE_UNITS * CLOCK_HZ)
    return {"scalar_per_clock_per_cu": per(rec["insts_salu"]), "vector_per_clock_per_cu": per(rec["insts_valu"]),
            "lds_per_clock_per_cu": per(rec["insts_lds"]), "peak_each": 1.0,
            "instructions_per_launch": rec["insts_salu"] + rec["insts_valu"] + rec["insts_lds"],
            "note": "instruction counts from the committed counter runs of this kernel, time from this run"}


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(batch, budget_s: float, threads: int):
    """The CPU oracle, as it stands, timed on bounded samples of the same batch: one thread on the
    first replays (extrapolated linearly), then all the host threads this process may use."""
    import oracle
    oracle.build()
    per_cells = batch.n_cells() / max(batch.n_replays, 1)
    hosts = batch.config["hosts_initial"]
    unit = "cell-events*hosts/s"
    # one replay first, to size the samples
    t0 = time.perf_counter()
    oracle.replay_batch(batch, replays=[0])
    one = max(time.perf_counter() - t0, 1e-6)
    # leg 1: one thread, the first min(n, 32) replays (fewer if they would not fit a third of the budget)
    n1 = int(max(1, min(batch.n_replays, 32, budget_s / 3 / one)))
    t0 = time.perf_counter()
    oracle.replay_batch(batch, replays=list(range(n1)))
    dt1 = time.perf_counter() - t0
    v1 = per_cells * n1 * hosts / dt1
    # leg 2: every host thread, replays striding over the threads; the whole batch if it fits the budget
    n = int(max(1, min(batch.n_replays, (2 * budget_s / 3) * threads / one)))
    idx = [int(i * batch.n_replays / n) for i in range(n)]
    t0 = time.perf_counter()
    oracle.replay_batch(batch, replays=idx, threads=threads)
    dt = time.perf_counter() - t0
    value = per_cells * n * hosts / dt
    return {"value": value, "unit": unit, "cores": threads, "kind": "oracle",
            "sample": f"{n} of {batch.n_replays} replays of {batch.name}, evenly spaced, "
                      f"{threads} thread(s), {dt:.1f} s",
            "host_cpus": os.cpu_count(), "cpu_model": cpu_model(),
            "threads_note": f"{threads} = min(hardware threads of the host, {GPU_BOX_CPU_SHARE}: the share of the "
                            f"box that goes with one GPU)",
            "one_core": {"value": v1, "unit": unit, "cores": 1,
                         "sample": f"first {n1} of {batch.n_replays} replays of {batch.name}, 1 thread, {dt1:.1f} s; "
                                   f"the whole batch would take {dt1 / n1 * batch.n_replays:.1f} s at this rate"}}


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
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "c4a", "c2b", "c4b", "c2l", "c4l"])
    ap.add_argument("--replays", type=int, default=None, help="truncate the batch (for quick looks)")
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time; 0 = skip")
    ap.add_argument("--cpu-threads", type=int, default=0, help="0 = all host threads this process may use")
    ap.add_argument("--hosts-in-lds", action="store_true", help="force the any-size kernel (comparison runs)")
    ap.add_argument("--generic-kernel", action="store_true", help="force the run-time-flags kernel (comparison runs)")
    ap.add_argument("--rounds", choices=["on", "off"], default=None, help="force the event-parallel rounds (comparison runs)")
    ap.add_argument("--one-wave", action="store_true", help="no helper waves on large clusters (comparison runs)")
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

    threads = args.cpu_threads or min(GPU_BOX_CPU_SHARE, os.cpu_count() or 1)
    t0 = time.perf_counter()
    batch = tracegen.workload(args.workload, n_replays=args.replays, workers=threads)
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
    default_shape = not (args.replays or args.hosts_in_lds or args.generic_kernel or args.rounds or args.one_wave)
    h = replay.Replay(batch.config, dev, hosts_in_lds=args.hosts_in_lds, generic_kernel=args.generic_kernel,
                      rounds=None if args.rounds is None else args.rounds == "on", one_wave=args.one_wave)
    info = h.launch_info()

    for _ in range(args.warmup):
        h.run()
    torch.cuda.synchronize()
    # The handle launches on torch's current stream, so events recorded there bracket every launch of
    # the timed region: marks[i] .. marks[i + 1] is launch i.
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()
        h.run()
    marks[args.steps].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dur = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
    last_ms = h.last_kernel_ms()            # the library's own HIP events around its last launch
    st = h.stats()
    assert (st["status"] == 0).all()
    h.close()
    copy_gbs = measured_copy_gbs(torch)
    floor_ns = replay.chain_floor_ns()

    ms_per_step = wall * 1e3 / args.steps
    cells = batch.n_cells()
    value = cells * batch.config["hosts_initial"] / (ms_per_step * 1e-3)
    alg_bytes = batch.algorithmic_bytes(replay.STATS_DTYPE.itemsize)
    avg_kernel_ms = sum(dur) / len(dur)
    achieved = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    ev_per_replay = batch.n_events() / max(batch.n_replays, 1)

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
                     "traffic": measured_traffic(args.workload) if default_shape else None,
                     "kernel": info["kernel"], "kernel_ms": avg_kernel_ms,
                     "kernel_ms_median": statistics.median(dur), "kernel_ms_last_by_library_events": last_ms,
                     "algorithmic_bytes": alg_bytes,
                     "ns_per_event_per_replay": avg_kernel_ms * 1e6 / ev_per_replay,
                     "issue": issue_rates(args.workload, avg_kernel_ms * 1e-3) if default_shape else None,
                     "chain_floor_ns": floor_ns,
                     "chain_floor_note": "one dependent event body (LDS row read, count, wave minimum, LDS write) on a "
                                         "lone wave; a replay cannot take a step in less"},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
