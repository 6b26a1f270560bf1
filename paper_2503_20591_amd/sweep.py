"""Policy study on the GPU replay: one batch answers "what does the subscription-ratio cap cost and save".

Every trace is replayed under every cap (the replays of a trace share its events in device memory),
once under the NotebookOS policy and once under the Batch baseline (the paper's "Baselines" section); the
Reservation baseline is a closed form that every replay reports. The rows put side by side what the
paper's evaluation plots: hosts provisioned against the cap (section "Subscription Ratio"), GPU-hours bound to
notebooks against Reservation (section "Resource Usage & Efficiency"), the interactivity delay against Batch
(section "Interactivity"), and the provider's margin under the billing model (section "Monetary Cost").

Marshalling and reporting only: all policy arithmetic runs in the HIP kernels.

    python -m paper_2503_20591_amd.sweep            # prints a table for a small synthetic study
"""
from __future__ import annotations

import argparse

import numpy as np

from . import replay, tracegen as tg

MS_PER_HOUR = 3_600_000.0


def study_batch(n_traces: int = 4, caps=(1000, 1500, 2000, 3000, 4000), sessions: int = 1000, cells: int = 60_000,
                hosts_initial: int = 16, hosts_max: int = 256, flags: int = tg.F_MIGRATE | tg.F_SCALE_OUT,
                **config) -> tg.TraceBatch:
    """``n_traces`` diurnal traces (the recipe of workload c4 at the given size, seeds 0..n-1), each
    replayed under every cap: replay ``t * len(caps) + j`` is trace ``t`` under ``caps[j]``."""
    kw = tg.recipe("c4")["kw"]
    traces = [tg.make_trace(seed, sessions, cells, **kw) for seed in range(n_traces)]
    cfg = tg.base_config(hosts_initial=hosts_initial, hosts_max=hosts_max, flags=flags, min_hosts=hosts_initial)
    cfg.update(config)
    tor = [t for t in range(n_traces) for _ in caps]
    return tg.pack(cfg, traces, tor, [int(c) for _ in range(n_traces) for c in caps], "study")


def _run(batch: tg.TraceBatch, dev: dict, price: int):
    h = replay.Replay(batch.config, dev)
    h.run()
    st, bill = h.stats(), h.billing(price)
    h.close()
    if (st["status"] != 0).any():
        raise RuntimeError("a replay ended with a non-zero status")
    return st, bill


def run_policies(batch: tg.TraceBatch, batch_start_delay_ms: int = 15_000,
                 price_micro_per_host_hour: int = 10_000_000, device: str = "cuda:0") -> list[dict]:
    """Replays ``batch`` under its own (NotebookOS) configuration and under the Batch baseline on the
    same cluster bounds; one row per (trace, cap)."""
    replay.load()
    dev = replay.upload(batch, device)
    nb, nb_bill = _run(batch, dev, price_micro_per_host_hour)
    as_batch = _with_config(batch, flags=tg.F_BATCH_MODE | (batch.config["flags"] & tg.F_SCALE_OUT),
                                 batch_start_delay_ms=batch_start_delay_ms)
    ba, _ = _run(as_batch, dev, price_micro_per_host_hour)
    G = batch.config["gpus_per_host"]
    rows = []
    for r in range(batch.n_replays):
        a, b = nb[r], ba[r]
        started = max(int(a["cells_started"]), 1)
        revenue = int(nb_bill["usage_revenue"][r]) + int(nb_bill["standby_revenue"][r])
        cost = int(nb_bill["provider_cost"][r])
        rows.append(dict(
            trace=int(batch.trace_of_replay[r]), cap=int(batch.cap_milli[r]) / 1000.0,
            peak_hosts=int(a["peak_hosts"]),
            provisioned_gpu_h=int(a["gpu_ms_provisioned"]) / MS_PER_HOUR,
            committed_gpu_h=int(a["gpu_ms_committed"]) / MS_PER_HOUR,
            reservation_gpu_h=int(a["reservation_gpu_ms"]) / MS_PER_HOUR,
            saved_vs_reservation=1.0 - int(a["gpu_ms_committed"]) / max(int(a["reservation_gpu_ms"]), 1),
            mean_delay_s=int(a["sum_delay_ms"]) / started / 1e3,
            immediate=int(a["cells_immediate"]) / started,
            migrations=int(a["migrations"]), aborted=int(a["cells_aborted"]), rejected=int(a["sessions_rejected"]),
            margin=(revenue - cost) / revenue if revenue > 0 else float("nan"),
            batch_peak_hosts=int(b["peak_hosts"]),
            batch_provisioned_gpu_h=int(b["gpu_ms_provisioned"]) / MS_PER_HOUR,
            batch_mean_delay_s=int(b["sum_delay_ms"]) / max(int(b["cells_started"]), 1) / 1e3,
            hosts_gpus=G))
    return rows


def _with_config(batch: tg.TraceBatch, **config) -> tg.TraceBatch:
    """The same traces and replays under a changed configuration."""
    import dataclasses
    return dataclasses.replace(batch, config=dict(batch.config, **config))


def format_table(rows: list[dict]) -> str:
    head = ["trace", "cap", "peak hosts", "prov. GPU-h", "bound GPU-h", "Reservation GPU-h", "saved", "delay s",
            "immediate", "migrations", "margin", "Batch hosts", "Batch delay s"]
    out = ["| " + " | ".join(head) + " |", "|" + "---|" * len(head)]
    for x in rows:
        out.append(f"| {x['trace']} | {x['cap']:.1f} | {x['peak_hosts']} | {x['provisioned_gpu_h']:.0f} | "
                   f"{x['committed_gpu_h']:.0f} | {x['reservation_gpu_h']:.0f} | {100 * x['saved_vs_reservation']:.1f} % | "
                   f"{x['mean_delay_s']:.2f} | {100 * x['immediate']:.1f} % | {x['migrations']} | {100 * x['margin']:.1f} % | "
                   f"{x['batch_peak_hosts']} | {x['batch_mean_delay_s']:.2f} |")
    return "\n".join(out)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--traces", type=int, default=2)
    ap.add_argument("--sessions", type=int, default=1000)
    ap.add_argument("--cells", type=int, default=60_000)
    ap.add_argument("--caps", default="1000,1500,2000,3000,4000", help="cap_milli values, comma separated")
    args = ap.parse_args()
    caps = [int(c) for c in args.caps.split(",")]
    print(format_table(run_policies(study_batch(args.traces, caps, args.sessions, args.cells))))


if __name__ == "__main__":
    main()
