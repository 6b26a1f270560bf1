"""CPU oracle of the NotebookOS policy replay -- TEST INFRASTRUCTURE, not product.

Thin ctypes loader around ``nbos_oracle.c`` (plain C, single-threaded, eager
discrete-event loop written from paper Sections 3.2.1-3.2.3, 3.3, 3.4.1, 3.4.2).
Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package. It imports nothing from the GPU library and shares no code with it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "nbos_oracle.c")
_SRC_BATCH = os.path.join(_DIR, "nbos_oracle_batch.c")
_LIB = os.path.join(_DIR, "libnbos_oracle.so")

F_MIGRATE, F_SCALE_OUT, F_SCALE_IN = 1, 2, 4
F_AUTOSCALE, F_DYNAMIC_SR, F_STICKY, F_BATCH, F_WARM_POOL, F_CLOSED_LOOP = 0x20, 0x40, 0x80, 0x100, 0x200, 0x400
EV_START, EV_CELL, EV_END = 0, 1, 2
(D_PLACE, D_PLACE_NEW, D_REJECT, D_START, D_MIGRATE, D_SCALE_CELL, D_ABORT, D_SCALE_IN,
 D_SCALE_AUTO, D_BATCH_START, D_BATCH_HOST, D_MIGRATE_WARM) = range(1, 13)


class _Params(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("hosts_initial", "hosts_max", "gpus_per_host")] + [
        ("flags", C.c_uint32)] + [(n, C.c_int32) for n in (
            "migration_delay_ms", "boot_delay_ms", "retry_interval_ms", "max_retries",
            "scale_interval_ms", "scale_in_idle_pct", "min_hosts", "cap_milli", "check",
            "autoscale_f_milli", "scaling_buffer_hosts", "batch_start_delay_ms",
            "warm_pool_per_host", "warm_migration_delay_ms", "prewarm_delay_ms")]


_U32 = ("n_decisions", "sessions_placed", "sessions_rejected", "cells_total", "cells_immediate",
        "cells_started", "cells_queued", "cells_aborted", "cells_dropped_busy",
        "cells_dropped_unplaced", "executor_reused", "migrations", "scale_out_hosts",
        "scale_in_hosts", "peak_hosts", "migrations_warm")
_I32 = ("max_delay_ms", "t_end_ms")
_I64 = ("sum_delay_ms", "sum_tct_ms", "gpu_ms_executed", "gpu_ms_committed",
        "gpu_ms_provisioned", "reservation_gpu_ms", "sub_gpu_ms", "replica_ms")


class _Result(C.Structure):
    _fields_ = ([(n, C.c_uint32) for n in _U32] + [(n, C.c_int32) for n in _I32] +
                [("delay_hist", C.c_uint32 * 32)] + [(n, C.c_int64) for n in _I64] +
                [("digest", C.c_uint64)])


class _Bill(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("provider_cost", "usage_revenue", "standby_revenue",
                                         "reservation_revenue")]


class _Final(C.Structure):
    _fields_ = [(n, C.POINTER(C.c_int32)) for n in (
        "host_state", "host_committed", "host_subscribed", "host_nrep", "sess_state", "sess_hosts")]


#: names of all result fields, in struct order (delay_hist is a list of 32)
RESULT_FIELDS = _U32 + _I32 + ("delay_hist",) + _I64 + ("digest",)

_lib = None


def build(force: bool = False, extra_cflags: tuple[str, ...] = (), out: str | None = None) -> str:
    """Compile the oracle with gcc. Returns the path of the shared object."""
    out = out or _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < max(
            os.path.getmtime(_SRC), os.path.getmtime(_SRC_BATCH), os.path.getmtime(os.path.join(_DIR, "nbos_oracle.h"))):
        cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", *extra_cflags,
               "-o", out, _SRC, _SRC_BATCH]
        subprocess.run(cmd, check=True, cwd=_DIR)
    return out


def _load(path: str | None = None):
    global _lib
    if path is None and _lib is not None:
        return _lib
    lib = C.CDLL(path or build())
    lib.orc_replay.restype = C.c_int
    lib.orc_replay.argtypes = [
        C.POINTER(_Params), C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
        C.c_int32, C.c_void_p, C.POINTER(_Result), C.c_void_p, C.c_int64, C.POINTER(_Final)]
    lib.orc_replay_batch.restype = C.c_int
    lib.orc_replay_batch.argtypes = lib.orc_replay.argtypes[:-1]
    lib.orc_sizeof_result.restype = C.c_int
    lib.orc_billing.restype = None
    lib.orc_billing.argtypes = [C.POINTER(_Result), C.c_int, C.c_int64, C.c_int, C.c_int, C.POINTER(_Bill)]
    assert lib.orc_sizeof_result() == C.sizeof(_Result)
    if path is None:
        _lib = lib
    return lib


def replay(cfg: dict, ev_time, ev_dur, ev_sk, sess_gpus, cap_milli: int, *, check: bool = False,
           want_log: bool = False, want_final: bool = False, lib_path: str | None = None) -> dict:
    """Replay ONE trace on one simulated cluster; returns the result fields as a dict.

    ``cfg`` holds hosts_initial, hosts_max, gpus_per_host, flags and the delay /
    retry / scale parameters (missing ones default to 0). Raises ValueError on a
    negative return of the C routine (``.args[1]`` is the code).
    """
    lib = _load(lib_path)
    ev_time = np.ascontiguousarray(ev_time, dtype=np.int32)
    ev_dur = np.ascontiguousarray(ev_dur, dtype=np.int32)
    ev_sk = np.ascontiguousarray(ev_sk, dtype=np.int32)
    sess_gpus = np.ascontiguousarray(sess_gpus, dtype=np.uint8)
    n_ev, n_s = int(ev_time.shape[0]), int(sess_gpus.shape[0])
    assert ev_dur.shape[0] == n_ev and ev_sk.shape[0] == n_ev
    p = _Params()
    for name, _ in _Params._fields_:
        if name in ("cap_milli", "check"):
            continue
        setattr(p, name, int(cfg.get(name, 0)))
    p.cap_milli = int(cap_milli)
    p.check = 1 if check else 0
    res = _Result()
    log = None
    log_cap = 0
    if want_log:
        log_cap = 3 * n_s + 2 * n_ev + 65536
        log = np.zeros(log_cap, dtype=np.uint64)
    fin = None
    keep = {}
    if want_final:
        fin = _Final()
        hm = int(cfg["hosts_max"])
        for name, n in (("host_state", hm), ("host_committed", hm), ("host_subscribed", hm),
                        ("host_nrep", hm), ("sess_state", max(n_s, 1)), ("sess_hosts", max(3 * n_s, 1))):
            keep[name] = np.zeros(n, dtype=np.int32)
            setattr(fin, name, keep[name].ctypes.data_as(C.POINTER(C.c_int32)))
    if p.flags & F_BATCH:        # the Batch baseline has a replay loop of its own (no final-state dump)
        rc = lib.orc_replay_batch(C.byref(p), n_ev, ev_time.ctypes.data, ev_dur.ctypes.data, ev_sk.ctypes.data,
                                  n_s, sess_gpus.ctypes.data, C.byref(res),
                                  log.ctypes.data if log is not None else None, log_cap)
    else:
        rc = lib.orc_replay(C.byref(p), n_ev, ev_time.ctypes.data, ev_dur.ctypes.data, ev_sk.ctypes.data,
                            n_s, sess_gpus.ctypes.data, C.byref(res),
                            log.ctypes.data if log is not None else None, log_cap,
                            C.byref(fin) if fin is not None else None)
    if rc != 0:
        raise ValueError(f"orc_replay failed with code {rc}", rc)
    out = {}
    for name in RESULT_FIELDS:
        v = getattr(res, name)
        out[name] = [int(x) for x in v] if name == "delay_hist" else int(v)
    if want_log:
        out["log"] = log[: min(out["n_decisions"], log_cap)].copy()
    if want_final:
        out["final"] = keep
    return out


def replay_batch(batch, replays=None, *, check: bool = False, threads: int = 1) -> list[dict]:
    """Replay several replays of a trace batch (see the trace generator's ``TraceBatch``)."""
    idx = list(range(batch.n_replays)) if replays is None else list(replays)

    def one(r):
        t = int(batch.trace_of_replay[r])
        a, b = int(batch.ev_offset[t]), int(batch.ev_offset[t + 1])
        sa, sb = int(batch.sess_offset[t]), int(batch.sess_offset[t + 1])
        return replay(batch.config, batch.ev_time[a:b], batch.ev_dur[a:b], batch.ev_sk[a:b],
                      batch.sess_gpus[sa:sb], int(batch.cap_milli[r]), check=check)

    if threads <= 1:
        return [one(r) for r in idx]
    from concurrent.futures import ThreadPoolExecutor
    _load()
    with ThreadPoolExecutor(max_workers=threads) as ex:   # ctypes releases the GIL in the C call
        return list(ex.map(one, idx))


def billing(result: dict, gpus_per_host: int, price_micro_per_host_hour: int, markup_pct: int = 115,
            standby_permille: int = 125, lib_path: str | None = None) -> dict:
    """Section "Monetary Cost" billing of one result dict (as returned by ``replay``), integer micro-dollars."""
    lib = _load(lib_path)
    res = _Result()
    for name in RESULT_FIELDS:
        if name == "delay_hist":
            for i, v in enumerate(result[name]):
                res.delay_hist[i] = v
        else:
            setattr(res, name, result[name])
    out = _Bill()
    lib.orc_billing(C.byref(res), int(gpus_per_host), int(price_micro_per_host_hour), int(markup_pct),
                    int(standby_permille), C.byref(out))
    return {n: int(getattr(out, n)) for n, _ in _Bill._fields_}


def decode(code: int) -> dict:
    """Split a decision code into its fields."""
    code = int(code)
    return {"host": code & 0x3FF, "slot": (code >> 10) & 3, "outcome": (code >> 12) & 0xF,
            "session": (code >> 16) & 0xFFFF, "time": code >> 32}
