"""ctypes binding of libnbos.so: argument marshalling only, every step runs in the HIP kernels.

    rp = Replay(config, device_inputs)     # nbos_replay_create
    rp.run()                               # nbos_replay_run (async on the stream)
    st = rp.stats()                        # nbos_replay_stats -> numpy structured array

``device_inputs`` maps the field names of ``nbos_inputs`` to torch CUDA tensors (kept alive by the
object); ``upload(batch)`` makes them from a host-side trace batch.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libnbos.so")

F_MIGRATE, F_SCALE_OUT, F_SCALE_IN, F_DECISION_LOG, F_HOSTS_IN_LDS = 1, 2, 4, 8, 16
F_AUTOSCALE, F_DYNAMIC_SR, F_STICKY_EXECUTOR, F_BATCH_MODE, F_WARM_POOL = 0x20, 0x40, 0x80, 0x100, 0x200
F_CLOSED_LOOP = 0x400
F_GENERIC_KERNEL, F_ROUNDS_OFF, F_ROUNDS_ON, F_ONE_WAVE = 0x800, 0x1000, 0x2000, 0x4000   # comparison runs: same results
E_ARG, E_RANGE, E_LIMIT, E_HIP, E_NOMEM, E_STATE = -1, -2, -3, -4, -5, -6

EXPORTS = ("nbos_replay_create", "nbos_replay_run", "nbos_replay_stats", "nbos_replay_decisions",
           "nbos_replay_billing", "nbos_replay_last_kernel_ms", "nbos_replay_launch_info", "nbos_replay_destroy",
           "nbos_strerror", "nbos_last_error_detail", "nbos_sizeof_stats", "nbos_replay_kernel_name",
           "nbos_chain_floor_ns", "nbos_replay_run_static")


class NbosConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_replays", C.c_int32), ("n_traces", C.c_int32),
                ("hosts_initial", C.c_int32), ("hosts_max", C.c_int32), ("gpus_per_host", C.c_int32),
                ("replicas", C.c_int32), ("flags", C.c_uint32), ("migration_delay_ms", C.c_int32),
                ("boot_delay_ms", C.c_int32), ("retry_interval_ms", C.c_int32), ("max_retries", C.c_int32),
                ("scale_interval_ms", C.c_int32), ("scale_in_idle_pct", C.c_int32), ("min_hosts", C.c_int32),
                ("autoscale_f_milli", C.c_int32), ("scaling_buffer_hosts", C.c_int32),
                ("batch_start_delay_ms", C.c_int32), ("warm_pool_per_host", C.c_int32),
                ("warm_migration_delay_ms", C.c_int32), ("prewarm_delay_ms", C.c_int32)]


_INPUT_FIELDS = ("ev_offset", "ev_time_ms", "ev_dur_ms", "ev_sess_kind", "sess_offset", "sess_gpus",
                 "trace_of_replay", "cap_milli")


class NbosBillingParams(C.Structure):
    _fields_ = [("price_micro_per_host_hour", C.c_int64), ("markup_pct", C.c_int32), ("standby_permille", C.c_int32)]


BILL_DTYPE = np.dtype([("provider_cost", "<i8"), ("usage_revenue", "<i8"), ("standby_revenue", "<i8"),
                       ("reservation_revenue", "<i8")])


class NbosInputs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _INPUT_FIELDS]


STATS_DTYPE = np.dtype(
    [("status", "<i4"), ("n_decisions", "<u4"), ("sessions_placed", "<u4"), ("sessions_rejected", "<u4"),
     ("cells_total", "<u4"), ("cells_immediate", "<u4"), ("cells_started", "<u4"), ("cells_queued", "<u4"),
     ("cells_aborted", "<u4"), ("cells_dropped_busy", "<u4"), ("cells_dropped_unplaced", "<u4"),
     ("executor_reused", "<u4"), ("migrations", "<u4"), ("scale_out_hosts", "<u4"), ("scale_in_hosts", "<u4"),
     ("peak_hosts", "<u4"), ("migrations_warm", "<u4"), ("max_delay_ms", "<i4"), ("t_end_ms", "<i4"), ("delay_hist", "<u4", (32,)),
     ("sum_delay_ms", "<i8"), ("sum_tct_ms", "<i8"), ("gpu_ms_executed", "<i8"), ("gpu_ms_committed", "<i8"),
     ("gpu_ms_provisioned", "<i8"), ("reservation_gpu_ms", "<i8"), ("sub_gpu_ms", "<i8"), ("replica_ms", "<i8"),
     ("digest", "<u8")],
    align=True)

_lib = None


class NbosError(RuntimeError):
    def __init__(self, code: int, what: str):
        detail = load().nbos_last_error_detail().decode() if code == E_HIP else ""
        super().__init__(f"{what}: {strerror(code)} ({code})" + (f": {detail}" if detail else ""))
        self.code = code


def load():
    """Load libnbos.so (built in-tree by ``build.build_library``). No fallback: raises if missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with paper_2503_20591_amd.build.build_library()")
    # torch first: the library has to share the HIP runtime that owns torch's device memory and streams
    # (loaded the other way round, the process holds two runtimes and this one finds no device)
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    lib.nbos_replay_create.restype = C.c_int32
    lib.nbos_replay_create.argtypes = [C.POINTER(NbosConfig), C.POINTER(NbosInputs), C.c_void_p,
                                       C.POINTER(C.c_void_p)]
    lib.nbos_replay_run.restype = C.c_int32
    lib.nbos_replay_run.argtypes = [C.c_void_p]
    lib.nbos_replay_stats.restype = C.c_int32
    lib.nbos_replay_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.nbos_replay_decisions.restype = C.c_int64
    lib.nbos_replay_decisions.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64]
    lib.nbos_replay_billing.restype = C.c_int32
    lib.nbos_replay_billing.argtypes = [C.c_void_p, C.POINTER(NbosBillingParams), C.c_int32, C.c_int32, C.c_void_p]
    lib.nbos_replay_last_kernel_ms.restype = C.c_int32
    lib.nbos_replay_last_kernel_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
    lib.nbos_replay_launch_info.restype = C.c_int32
    lib.nbos_replay_launch_info.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                            C.POINTER(C.c_int32)]
    lib.nbos_replay_destroy.restype = None
    lib.nbos_replay_destroy.argtypes = [C.c_void_p]
    lib.nbos_strerror.restype = C.c_char_p
    lib.nbos_strerror.argtypes = [C.c_int32]
    lib.nbos_last_error_detail.restype = C.c_char_p
    lib.nbos_last_error_detail.argtypes = []
    lib.nbos_sizeof_stats.restype = C.c_int32
    lib.nbos_replay_kernel_name.restype = C.c_char_p
    lib.nbos_replay_kernel_name.argtypes = [C.c_void_p]
    lib.nbos_replay_run_static.restype = C.c_int32
    lib.nbos_replay_run_static.argtypes = [C.POINTER(NbosConfig), C.POINTER(NbosInputs), C.c_int32, C.c_void_p, C.c_void_p]
    lib.nbos_chain_floor_ns.restype = C.c_int32
    lib.nbos_chain_floor_ns.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_float)]
    if lib.nbos_sizeof_stats() != STATS_DTYPE.itemsize:
        raise RuntimeError("nbos_stats layout mismatch between the binding and libnbos.so")
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().nbos_strerror(int(code)).decode()


def make_config(cfg: dict, n_replays: int, n_traces: int, extra_flags: int = 0) -> NbosConfig:
    c = NbosConfig()
    c.struct_size = C.sizeof(NbosConfig)
    c.n_replays, c.n_traces = int(n_replays), int(n_traces)
    c.replicas = int(cfg.get("replicas", 3))
    for name in ("hosts_initial", "hosts_max", "gpus_per_host", "migration_delay_ms", "boot_delay_ms",
                 "retry_interval_ms", "max_retries", "scale_interval_ms", "scale_in_idle_pct", "min_hosts",
                 "autoscale_f_milli", "scaling_buffer_hosts", "batch_start_delay_ms", "warm_pool_per_host",
                 "warm_migration_delay_ms", "prewarm_delay_ms"):
        setattr(c, name, int(cfg.get(name, 0)))
    c.flags = int(cfg.get("flags", 0)) | int(extra_flags)
    return c


def upload(batch, device="cuda:0") -> dict:
    """Copy a host-side trace batch into device tensors named after the nbos_inputs fields."""
    import torch
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
    return {"ev_offset": t(batch.ev_offset.astype(np.int64)), "ev_time_ms": t(batch.ev_time),
            "ev_dur_ms": t(batch.ev_dur), "ev_sess_kind": t(batch.ev_sk),
            "sess_offset": t(batch.sess_offset.astype(np.int32)), "sess_gpus": t(batch.sess_gpus),
            "trace_of_replay": t(batch.trace_of_replay.astype(np.int32)),
            "cap_milli": t(batch.cap_milli.astype(np.int32))}


class Replay:
    """Owns one nbos_replay handle. ``inputs``: dict of torch CUDA tensors (borrowed by the library,
    kept referenced here). ``stream``: a torch.cuda.Stream or None for the current stream."""

    def __init__(self, cfg: dict, inputs: dict, n_replays: int | None = None, n_traces: int | None = None,
                 stream=None, decision_log: bool = False, hosts_in_lds: bool = False,
                 generic_kernel: bool = False, rounds: bool | None = None, one_wave: bool = False):
        import torch
        lib = load()
        self._lib = lib
        self._keep = dict(inputs)
        n_replays = int(inputs["trace_of_replay"].numel()) if n_replays is None else n_replays
        n_traces = int(inputs["ev_offset"].numel()) - 1 if n_traces is None else n_traces
        self.n_replays = n_replays
        self.config = make_config(cfg, n_replays, n_traces, (F_DECISION_LOG if decision_log else 0)
                                  | (F_HOSTS_IN_LDS if hosts_in_lds else 0)
                                  | (F_GENERIC_KERNEL if generic_kernel else 0) | (F_ONE_WAVE if one_wave else 0)
                                  | (0 if rounds is None else F_ROUNDS_ON if rounds else F_ROUNDS_OFF))
        ins = NbosInputs()
        for name in _INPUT_FIELDS:
            ten = inputs[name]
            if not ten.is_cuda or not ten.is_contiguous():
                raise ValueError(f"{name} must be a contiguous CUDA tensor")
            setattr(ins, name, ten.data_ptr() if ten.numel() else None)
        self._stream = stream if stream is not None else torch.cuda.current_stream(inputs["cap_milli"].device)
        h = C.c_void_p()
        with torch.cuda.device(inputs["cap_milli"].device):
            rc = lib.nbos_replay_create(C.byref(self.config), C.byref(ins), C.c_void_p(self._stream.cuda_stream),
                                        C.byref(h))
        if rc != 0:
            raise NbosError(rc, "nbos_replay_create")
        self._h = h

    def run(self):
        rc = self._lib.nbos_replay_run(self._h)
        if rc != 0:
            raise NbosError(rc, "nbos_replay_run")

    def stats(self, first: int = 0, count: int | None = None) -> np.ndarray:
        count = self.n_replays - first if count is None else count
        out = np.zeros(count, dtype=STATS_DTYPE)
        rc = self._lib.nbos_replay_stats(self._h, first, count, out.ctypes.data)
        if rc != 0:
            raise NbosError(rc, "nbos_replay_stats")
        return out

    def decisions(self, replay: int, cap: int = 1 << 22) -> np.ndarray:
        buf = np.zeros(cap, dtype=np.uint64)
        n = self._lib.nbos_replay_decisions(self._h, replay, buf.ctypes.data, cap)
        if n < 0:
            raise NbosError(int(n), "nbos_replay_decisions")
        return buf[: min(n, cap)].copy()

    def billing(self, price_micro_per_host_hour: int, markup_pct: int = 115, standby_permille: int = 125,
                first: int = 0, count: int | None = None) -> np.ndarray:
        """Bills (structured array of BILL_DTYPE) of the last run, computed on the device."""
        count = self.n_replays - first if count is None else count
        bp = NbosBillingParams(int(price_micro_per_host_hour), int(markup_pct), int(standby_permille))
        out = np.zeros(max(count, 0), dtype=BILL_DTYPE)
        rc = self._lib.nbos_replay_billing(self._h, C.byref(bp), first, count, out.ctypes.data)
        if rc != 0:
            raise NbosError(rc, "nbos_replay_billing")
        return out

    def last_kernel_ms(self) -> float:
        ms = C.c_float()
        rc = self._lib.nbos_replay_last_kernel_ms(self._h, C.byref(ms))
        if rc != 0:
            raise NbosError(rc, "nbos_replay_last_kernel_ms")
        return float(ms.value)

    def launch_info(self) -> dict:
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        self._lib.nbos_replay_launch_info(self._h, C.byref(a), C.byref(b), C.byref(c))
        return {"lds_bytes": a.value, "threads_per_group": b.value, "groups": c.value,
                "kernel": self._lib.nbos_replay_kernel_name(self._h).decode()}

    def close(self):
        if getattr(self, "_h", None):
            self._lib.nbos_replay_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def run_static(cfg: dict, inputs: dict, max_sessions_per_trace: int, stats_out, stream=None) -> None:
    """nbos_replay_run_static: one pass enqueued on torch's current stream without any allocation by the
    library. ``stats_out``: a CUDA uint8 tensor of n_replays * STATS_DTYPE.itemsize bytes (the caller's);
    read it with ``stats_from_tensor`` after synchronising."""
    import torch
    lib = load()
    n_replays = int(inputs["trace_of_replay"].numel())
    c = make_config(cfg, n_replays, int(inputs["ev_offset"].numel()) - 1)
    ins = NbosInputs()
    for name in _INPUT_FIELDS:
        ten = inputs[name]
        if not ten.is_cuda or not ten.is_contiguous():
            raise ValueError(f"{name} must be a contiguous CUDA tensor")
        setattr(ins, name, ten.data_ptr() if ten.numel() else None)
    if not stats_out.is_cuda or stats_out.numel() * stats_out.element_size() < n_replays * STATS_DTYPE.itemsize:
        raise ValueError("stats_out must be a CUDA tensor with room for n_replays records")
    st = stream if stream is not None else torch.cuda.current_stream(stats_out.device)
    with torch.cuda.device(stats_out.device):
        rc = lib.nbos_replay_run_static(C.byref(c), C.byref(ins), int(max_sessions_per_trace),
                                        C.c_void_p(st.cuda_stream), C.c_void_p(stats_out.data_ptr()))
    if rc != 0:
        raise NbosError(rc, "nbos_replay_run_static")


def stats_from_tensor(stats_out, n_replays: int) -> np.ndarray:
    """The records a run_static call left in ``stats_out`` (synchronises through the copy to the host)."""
    raw = stats_out.view(-1).cpu().numpy().view(np.uint8)[: n_replays * STATS_DTYPE.itemsize]
    return raw.view(STATS_DTYPE).copy()


def chain_floor_ns(iters: int = 200_000, stream=None) -> float:
    """nbos_chain_floor_ns on torch's current stream: ns per iteration of the shortest event body."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    ns = C.c_float()
    rc = load().nbos_chain_floor_ns(C.c_void_p(st.cuda_stream), int(iters), C.byref(ns))
    if rc != 0:
        raise NbosError(rc, "nbos_chain_floor_ns")
    return float(ns.value)


DECISION_NAMES = {1: "PLACE", 2: "PLACE_NEW", 3: "REJECT", 4: "START", 5: "MIGRATE", 6: "SCALE_CELL", 7: "ABORT",
                  8: "SCALE_IN", 9: "SCALE_AUTO", 10: "BATCH_START", 11: "BATCH_HOST", 12: "MIGRATE_WARM"}


def decode_decision(code: int) -> dict:
    """The fields of one decision code (layout of nbos.h: host | slot << 10 | outcome << 12 |
    session << 16 | time << 32)."""
    code = int(code)
    outcome = (code >> 12) & 0xF
    return {"time_ms": code >> 32, "session": (code >> 16) & 0xFFFF, "outcome": outcome,
            "name": DECISION_NAMES.get(outcome, "?"), "slot": (code >> 10) & 3, "host": code & 0x3FF}


def stats_to_dict(row) -> dict:
    """One stats record as plain Python ints (delay_hist as a list)."""
    return {n: ([int(x) for x in row[n]] if n == "delay_hist" else int(row[n])) for n in STATS_DTYPE.names}
