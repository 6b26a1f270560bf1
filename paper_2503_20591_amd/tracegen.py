"""Seeded synthetic notebook-session traces (inputs only; none of the policy's arithmetic).

The paper measured on a private trace of an internal notebook platform
(its section "Real-World IDLT Workload Analysis": 545,467 training events, 15 s granularity). That trace is not
public, so these generators stand in for it and take its shape: per-session
streams, one cell at a time per session (Observation 2), short tasks (median
2 min, p75 5 min), long idle gaps (median 5 min), GPU requests in powers of two
on 8-GPU servers (the evaluation's "Setup" section).

A trace is three int32 arrays sorted by time (time_ms, dur_ms, session|kind<<24)
plus one GPU request per session. Trace ``k`` depends only on its own seed, so a
batch is reproducible trace by trace. Randomness: numpy's counter-based Philox.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ProcessPoolExecutor

import numpy as np

EV_START, EV_CELL, EV_END = 0, 1, 2
F_MIGRATE, F_SCALE_OUT, F_SCALE_IN = 1, 2, 4
F_AUTOSCALE, F_DYNAMIC_SR, F_STICKY_EXECUTOR, F_BATCH_MODE, F_WARM_POOL = 0x20, 0x40, 0x80, 0x100, 0x200
F_CLOSED_LOOP = 0x400

MAX_DUR_MS = 86_400_000          # a cell or an idle gap is at most 24 h
MAX_TIME_MS = 1_900_000_000      # arrivals are clipped here so finish times stay in int32
DAY_MS = 86_400_000


@dataclasses.dataclass
class TraceBatch:
    """Host-side (numpy) image of the replay inputs."""
    config: dict                  # hosts_initial, hosts_max, gpus_per_host, flags, delays...
    ev_offset: np.ndarray         # int64 [n_traces+1]
    ev_time: np.ndarray           # int32
    ev_dur: np.ndarray            # int32
    ev_sk: np.ndarray             # int32  session | kind << 24
    sess_offset: np.ndarray       # int32 [n_traces+1]
    sess_gpus: np.ndarray         # uint8
    trace_of_replay: np.ndarray   # int32 [n_replays]
    cap_milli: np.ndarray         # int32 [n_replays]
    name: str = ""

    @property
    def n_replays(self) -> int:
        return int(self.trace_of_replay.shape[0])

    @property
    def n_traces(self) -> int:
        return int(self.ev_offset.shape[0]) - 1

    def n_cells(self) -> int:
        """Cell events summed over replays (a trace shared by k replays counts k times)."""
        kinds = self.ev_sk.view(np.uint32) >> 24
        c = np.concatenate([np.zeros(1, np.int64), np.cumsum(kinds == EV_CELL, dtype=np.int64)])
        per_trace = c[self.ev_offset[1:]] - c[self.ev_offset[:-1]]
        return int(per_trace[self.trace_of_replay].sum())

    def n_events(self) -> int:
        per_trace = np.diff(self.ev_offset)
        return int(per_trace[self.trace_of_replay].sum())

    def algorithmic_bytes(self, stats_bytes: int) -> int:
        """What the method must move: 12 B per event (time, duration, session | kind) + 1 B per session
        + 8 B per replay read, one stats record written. The same for every mode: what a kernel moves
        beyond that (chain records and cursors of the closed loop, queued durations) is scratch traffic."""
        ev = np.diff(self.ev_offset)[self.trace_of_replay].sum()
        ss = np.diff(self.sess_offset)[self.trace_of_replay].sum()
        return int(12 * ev + ss + (8 + stats_bytes) * self.n_replays)


# ---- samplers: float64 seconds -> integer milliseconds ---------------------------------------

def _to_ms(sec: np.ndarray) -> np.ndarray:
    return np.clip(np.floor(sec * 1000.0), 1, MAX_DUR_MS).astype(np.int64)


def exp_ms(rng, mean_s, shape):
    return _to_ms(-mean_s * np.log1p(-rng.random(shape)))


def lognormal_ms(rng, median_s, sigma, shape):
    return _to_ms(np.exp(math.log(median_s) + sigma * rng.standard_normal(shape)))


def pareto_ms(rng, alpha, xmin_s, shape):
    return _to_ms(xmin_s * np.power(1.0 - rng.random(shape), -1.0 / alpha))


def gpus_uniform(rng, n):
    return np.array([1, 2, 4, 8], np.uint8)[rng.integers(0, 4, n)]


def gpus_weighted(rng, n):
    """1:0.5  2:0.25  4:0.15  8:0.1"""
    u = rng.random(n)
    return np.where(u < 0.5, 1, np.where(u < 0.75, 2, np.where(u < 0.9, 4, 8))).astype(np.uint8)


# ---- one trace ---------------------------------------------------------------------------------

def make_trace(seed: int, n_sessions: int, n_cells: int, *, ramp_ms: int, gpus, gap, dur,
               with_end: bool = False, diurnal: bool = False, mmpp=None):
    """One time-sorted trace.

    Each session s starts at U[0, ramp), then repeats {wait gap; submit a cell of length dur;
    wait for its nominal end}. Session s gets floor(E/N) cells (+1 for the first E mod N).
    ``gap(rng, shape)`` / ``dur(rng, shape)`` return int64 ms. ``diurnal`` divides every gap by
    m(t) = 1 + 0.5 sin(2 pi t / 24 h) evaluated at the time the gap begins. ``mmpp`` =
    (mean_fast_s, mean_slow_s, p_switch) replaces ``gap`` by a per-session two-state process.
    Events are merged by (time, session id, order within the session).
    """
    rng = np.random.Generator(np.random.Philox(key=seed))
    N, E = n_sessions, n_cells
    M = -(-E // N) if N else 0
    per = np.full(N, E // N if N else 0, np.int64)
    per[: (E % N if N else 0)] += 1
    g = gpus(rng, N)
    start = np.floor(rng.random(N) * ramp_ms).astype(np.int64)
    d = dur(rng, (N, M))
    if mmpp is not None:
        fast, slow, p_sw = mmpp
        state = np.cumsum(rng.random((N, M)) < p_sw, axis=1) & 1
        gp = np.where(state == 0, exp_ms(rng, fast, (N, M)), exp_ms(rng, slow, (N, M)))
    else:
        gp = gap(rng, (N, M))
    if diurnal:
        t = start.copy()
        tc = np.empty((N, M), np.int64)
        for k in range(M):
            m = 1.0 + 0.5 * np.sin(2.0 * math.pi * (t % DAY_MS) / DAY_MS)
            gk = np.clip(np.floor(gp[:, k] / m), 1, MAX_DUR_MS).astype(np.int64)
            tc[:, k] = t + gk
            t = tc[:, k] + d[:, k]
    else:
        tc = start[:, None] + np.cumsum(gp + d, axis=1) - d
    live = np.arange(M)[None, :] < per[:, None]
    sid = np.broadcast_to(np.arange(N, dtype=np.int64)[:, None], (N, M))
    seq = np.broadcast_to(np.arange(1, M + 1, dtype=np.int64)[None, :], (N, M))
    times = [start, tc[live]]
    durs = [np.zeros(N, np.int64), d[live]]
    sids = [np.arange(N, dtype=np.int64), sid[live]]
    seqs = [np.zeros(N, np.int64), seq[live]]
    kinds = [np.full(N, EV_START, np.int64), np.full(int(live.sum()), EV_CELL, np.int64)]
    if with_end:
        last = np.maximum(per - 1, 0)
        t_end = np.where(per > 0, tc[np.arange(N), last] + d[np.arange(N), last], start) if M else start
        times.append(t_end); durs.append(np.zeros(N, np.int64))
        sids.append(np.arange(N, dtype=np.int64)); seqs.append(np.full(N, M + 1, np.int64))
        kinds.append(np.full(N, EV_END, np.int64))
    t_all = np.minimum(np.concatenate(times), MAX_TIME_MS)
    s_all = np.concatenate(sids)
    key = (t_all << 32) | (s_all << 16) | np.concatenate(seqs)
    order = np.argsort(key, kind="stable")
    ev_time = t_all[order].astype(np.int32)
    ev_dur = np.concatenate(durs)[order].astype(np.int32)
    ev_sk = (s_all[order] | (np.concatenate(kinds)[order] << 24)).astype(np.int32)
    return ev_time, ev_dur, ev_sk, g


def _pack(config, traces, trace_of_replay, cap_milli, name) -> TraceBatch:
    ev_off = np.zeros(len(traces) + 1, np.int64)
    s_off = np.zeros(len(traces) + 1, np.int32)
    for i, (t, _, _, g) in enumerate(traces):
        ev_off[i + 1] = ev_off[i] + len(t)
        s_off[i + 1] = s_off[i] + len(g)
    cat = (lambda k, dt: np.concatenate([tr[k] for tr in traces]).astype(dt)
           if traces else np.zeros(0, dt))
    return TraceBatch(config=dict(config), ev_offset=ev_off, ev_time=cat(0, np.int32),
                      ev_dur=cat(1, np.int32), ev_sk=cat(2, np.int32), sess_offset=s_off,
                      sess_gpus=cat(3, np.uint8),
                      trace_of_replay=np.asarray(trace_of_replay, np.int32),
                      cap_milli=np.asarray(cap_milli, np.int32), name=name)


def _base_config(**kw) -> dict:
    cfg = dict(hosts_initial=8, hosts_max=8, gpus_per_host=8, flags=0, migration_delay_ms=15_000,
               boot_delay_ms=60_000, retry_interval_ms=10_000, max_retries=6,
               scale_interval_ms=60_000, scale_in_idle_pct=10, min_hosts=0,
               autoscale_f_milli=0, scaling_buffer_hosts=0, batch_start_delay_ms=0,
               warm_pool_per_host=0, warm_migration_delay_ms=0, prewarm_delay_ms=0)
    cfg.update(kw)
    return cfg


# ---- the five named workloads ------------------------------------------------------------------
# Each entry: config, sessions, cells per replay, trace recipe, cap rule. Values not fixed by the
# workload statement (ramp, unlisted distributions) are choices of this generator.

def _recipe(name: str):
    if name == "c1":   # 1 replay, 8 hosts, no migration, no autoscaling
        return dict(replays=1, cfg=_base_config(hosts_initial=8, hosts_max=8, flags=0),
                    N=50, E=2_000,
                    kw=dict(ramp_ms=600_000, gpus=gpus_uniform,
                            gap=lambda r, s: exp_ms(r, 60.0, s),
                            dur=lambda r, s: lognormal_ms(r, 30.0, 1.0, s)),
                    cap=lambda i, n: 2000)
    if name == "c2":   # cap swept 1.0-3.0 evenly, migration on
        return dict(replays=1024, cfg=_base_config(hosts_initial=30, hosts_max=30, flags=F_MIGRATE),
                    N=400, E=50_000,
                    kw=dict(ramp_ms=3_600_000, gpus=gpus_uniform,
                            gap=lambda r, s: pareto_ms(r, 1.5, 10.0, s),
                            dur=lambda r, s: lognormal_ms(r, 60.0, 1.2, s)),
                    cap=lambda i, n: 1000 + (2000 * i) // max(n - 1, 1))
    if name == "c3":   # heavy-tailed durations, caps {1.5, 2, 3, 4}, migration delay 15 s
        return dict(replays=4096, cfg=_base_config(hosts_initial=64, hosts_max=64, flags=F_MIGRATE),
                    N=1000, E=100_000,
                    kw=dict(ramp_ms=3_600_000, gpus=gpus_weighted,
                            gap=lambda r, s: pareto_ms(r, 1.5, 10.0, s),
                            dur=lambda r, s: pareto_ms(r, 1.3, 5.0, s)),
                    cap=lambda i, n: (1500, 2000, 3000, 4000)[i % 4])
    if name == "c4":   # diurnal arrivals, scale-out to 768 hosts, scale-in, END events
        return dict(replays=256,
                    cfg=_base_config(hosts_initial=512, hosts_max=768,
                                     flags=F_MIGRATE | F_SCALE_OUT | F_SCALE_IN, min_hosts=512),
                    N=8000, E=500_000,
                    kw=dict(ramp_ms=DAY_MS, gpus=gpus_weighted, diurnal=True, with_end=True,
                            gap=lambda r, s: 240_000 + lognormal_ms(r, 60.0, 2.06, s),
                            dur=lambda r, s: lognormal_ms(r, 120.0, 1.36, s)),
                    cap=lambda i, n: 2000)
    if name == "c5":   # occupancy stress: bursty two-state arrivals, scale-out to 24 hosts
        return dict(replays=16384,
                    cfg=_base_config(hosts_initial=16, hosts_max=24, flags=F_MIGRATE | F_SCALE_OUT),
                    N=120, E=20_000,
                    kw=dict(ramp_ms=600_000, gpus=gpus_uniform, mmpp=(10.0, 300.0, 0.1), gap=None,
                            dur=lambda r, s: lognormal_ms(r, 30.0, 1.0, s)),
                    cap=lambda i, n: 1000 + int(np.random.Generator(
                        np.random.Philox(key=0xCA9, counter=i)).integers(0, 3001)))
    if name == "c4a":  # the c4 traces with the cluster sized by the periodic auto-scaler alone
        # (Section 3.4.2: f = 1.05): 256 hosts at the start, a scaling buffer of 32 hosts, releases
        # down to 128 hosts, no scale-out on failed placement, cap 4.0 plus the dynamic limit
        rc = _recipe("c4")
        rc["cfg"] = dict(rc["cfg"], hosts_initial=256, min_hosts=128,
                         flags=F_MIGRATE | F_SCALE_IN | F_AUTOSCALE | F_DYNAMIC_SR,
                         autoscale_f_milli=1050, scaling_buffer_hosts=32)
        rc["cap"] = lambda i, n: 4000
        return rc
    if name in ("c2b", "c4b"):  # the c2 / c4 traces under the Batch baseline (the paper's "Baselines" section): a container
        # per cell (15 s to start, the GPUs already held), first come first served, fixed cluster
        rc = _recipe(name[:2])
        rc["cfg"] = dict(rc["cfg"], flags=F_BATCH_MODE, hosts_max=rc["cfg"]["hosts_initial"], batch_start_delay_ms=15_000)
        return rc
    if name in ("c2l", "c4l"):  # the c2 / c4 traces read as closed loops (the section "Interactive Deep Learning Training": a user submits the
        # next cell a think time after the previous one is over); c4l without the periodic scale-in
        rc = _recipe(name[:2])
        rc["cfg"] = dict(rc["cfg"], flags=(rc["cfg"]["flags"] & ~F_SCALE_IN) | F_CLOSED_LOOP)
        return rc
    raise KeyError(name)


# public names for building batches of one's own (policy studies, tests)
pack, base_config, recipe = _pack, _base_config, _recipe

WORKLOADS = ("c1", "c2", "c3", "c4", "c5", "c4a", "c2b", "c4b", "c2l", "c4l")


def _gen_range(args):
    name, lo, hi = args
    rc = _recipe(name)
    return [make_trace(seed, rc["N"], rc["E"], **rc["kw"]) for seed in range(lo, hi)]


def workload(name: str, n_replays: int | None = None, workers: int = 1) -> TraceBatch:
    """Named workload; trace seed = replay index. ``n_replays`` truncates the batch (the cap of
    replay i is still computed for the full batch size, so replay i is the same replay)."""
    rc = _recipe(name)
    full = rc["replays"]
    n = full if n_replays is None else min(int(n_replays), full)
    if workers > 1 and n >= 4 * workers:
        step = -(-n // (workers * 4))
        jobs = [(name, lo, min(lo + step, n)) for lo in range(0, n, step)]
        with ProcessPoolExecutor(max_workers=workers) as ex:
            traces = [t for part in ex.map(_gen_range, jobs) for t in part]
    else:
        traces = _gen_range((name, 0, n))
    caps = [rc["cap"](i, full) for i in range(n)]
    return _pack(rc["cfg"], traces, np.arange(n), caps, name)


# ---- small randomized cases for parity fuzzing -------------------------------------------------

def random_case(seed: int, n_replays: int = 4, policy_flags: bool = False) -> TraceBatch:
    """A small batch with randomly drawn cluster shape, flags, delays and load, including END
    events, repeated START / END events, and replays that share a trace. ``policy_flags`` adds
    the periodic auto-scaler, the dynamic subscription-ratio limit with low caps and / or the sticky-executor
    election."""
    rng = np.random.Generator(np.random.Philox(key=0x5EED0000 + seed))
    G = int(rng.choice([1, 2, 4, 8, 8, 8]))
    h0 = int(rng.integers(1, 20)) if rng.random() < 0.8 else int(rng.integers(60, 140))
    flags = int(rng.integers(0, 8))
    hmax = h0 + (int(rng.integers(0, 12)) if flags & F_SCALE_OUT else 0)
    cfg = _base_config(
        hosts_initial=h0, hosts_max=hmax, gpus_per_host=G, flags=flags,
        migration_delay_ms=int(rng.choice([0, 1, 500, 15_000])),
        boot_delay_ms=int(rng.choice([0, 1, 2_000, 60_000])),
        retry_interval_ms=int(rng.choice([1, 700, 10_000])),
        max_retries=int(rng.integers(0, 7)),
        scale_interval_ms=int(rng.choice([1_000, 7_000, 60_000])),
        scale_in_idle_pct=int(rng.choice([0, 10, 50, 100])),
        min_hosts=int(rng.integers(0, h0 + 1)))
    n_traces = int(rng.integers(1, n_replays + 1))
    load = float(rng.choice([0.3, 1.0, 3.0, 10.0]))
    traces = []
    for k in range(n_traces):
        N = int(rng.integers(1, 60))
        E = int(rng.integers(0, 700))
        gsel = (lambda r, n, G=G: np.minimum(gpus_uniform(r, n), G).astype(np.uint8))
        tr = make_trace(int(rng.integers(0, 2**31)), N, E, ramp_ms=int(rng.choice([1, 5_000, 300_000])),
                        gpus=gsel, gap=lambda r, s, load=load: exp_ms(r, 20.0 / load, s),
                        dur=lambda r, s: lognormal_ms(r, 15.0, 1.0, s),
                        with_end=bool(rng.random() < 0.6))
        t, d, sk, g = tr
        if len(t) and rng.random() < 0.5:      # sprinkle extra START / END / early CELL events
            m = int(rng.integers(1, 8))
            pos = np.sort(rng.integers(0, len(t), m))
            t = np.insert(t, pos, t[pos])
            d = np.insert(d, pos, np.maximum(d[pos], 1))
            extra = (rng.integers(0, N, m) | (rng.integers(0, 3, m) << 24)).astype(np.int32)
            sk = np.insert(sk, pos, extra)
        traces.append((t, d, sk, g))
    tor = rng.integers(0, n_traces, n_replays)
    caps = rng.choice([300, 333, 667, 1000, 1500, 2000, 3000, 4000, 100000], n_replays)
    if policy_flags:
        # the periodic auto-scaler and the dynamic limit, drawn from a stream of their own so that
        # the case is otherwise the same as without them
        r2 = np.random.Generator(np.random.Philox(key=0xA5CA1E00 + seed))
        extra = int(r2.choice([F_AUTOSCALE, F_DYNAMIC_SR, F_AUTOSCALE | F_DYNAMIC_SR, F_STICKY_EXECUTOR,
                               F_STICKY_EXECUTOR | F_AUTOSCALE | F_DYNAMIC_SR]))
        cfg["flags"] |= extra
        if extra & F_AUTOSCALE:
            cfg["hosts_max"] = max(cfg["hosts_max"], h0 + int(r2.integers(0, 12)))
            cfg["autoscale_f_milli"] = int(r2.choice([0, 1050, 1050, 2000, 8000]))
            cfg["scaling_buffer_hosts"] = int(r2.choice([0, 0, 1, 3]))
        if extra & F_DYNAMIC_SR:
            caps = r2.choice([20, 50, 100, 200, 334, 1000], n_replays)
        if r2.random() < 0.5:          # pre-warmed containers for migrations
            cfg["flags"] |= F_WARM_POOL | F_MIGRATE
            cfg["warm_pool_per_host"] = int(r2.integers(1, 5))
            cfg["warm_migration_delay_ms"] = int(r2.choice([0, 100, 2_000]))
            cfg["prewarm_delay_ms"] = int(r2.choice([0, 5_000, 60_000, 10_000_000]))
    return _pack(cfg, traces, tor, caps, f"random{seed}")
