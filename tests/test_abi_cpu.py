"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2503_20591_amd import replay

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(replay._LIB_PATH):
        from paper_2503_20591_amd.build import build_library
        build_library()
    return replay.load()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "nbos.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(nbos_[a-z_]+)\s*\(", hdr))
    assert declared == set(replay.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_sizes(lib):
    assert lib.nbos_sizeof_stats() == replay.STATS_DTYPE.itemsize == 280
    assert C.sizeof(replay.NbosConfig) == 21 * 4
    assert C.sizeof(replay.NbosInputs) == 8 * 8
    assert C.sizeof(replay.NbosBillingParams) == 16 and replay.BILL_DTYPE.itemsize == 32


def test_strerror(lib):
    assert replay.strerror(0) == "ok"
    seen = {replay.strerror(c) for c in range(-6, 1)}
    assert len(seen) == 7 and replay.strerror(-99) == "unknown status"


def _cfg(**kw):
    base = dict(hosts_initial=4, hosts_max=4, gpus_per_host=8, flags=0, migration_delay_ms=0, boot_delay_ms=0,
                retry_interval_ms=1000, max_retries=3, scale_interval_ms=1000, scale_in_idle_pct=10, min_hosts=0)
    base.update(kw)
    return base


def _create(lib, cfg, n_replays=1, n_traces=1, inputs=True, struct_size=None, out=True):
    c = replay.make_config(cfg, n_replays, n_traces)
    if struct_size is not None:
        c.struct_size = struct_size
    ins = replay.NbosInputs()
    h = C.c_void_p()
    rc = lib.nbos_replay_create(C.byref(c), C.byref(ins) if inputs else None, None, C.byref(h) if out else None)
    if rc == 0:
        lib.nbos_replay_destroy(h)
    return rc


@pytest.mark.parametrize("bad", [
    dict(replicas=2), dict(gpus_per_host=0), dict(gpus_per_host=9), dict(hosts_initial=0),
    dict(hosts_max=3), dict(migration_delay_ms=-1), dict(boot_delay_ms=-1), dict(retry_interval_ms=0),
    dict(max_retries=16), dict(max_retries=-1), dict(flags=0x404), dict(flags=0x8000), dict(flags=0x200), dict(flags=0x200, warm_pool_per_host=5), dict(flags=0x300, warm_pool_per_host=1),
    dict(flags=0x200, warm_pool_per_host=1, prewarm_delay_ms=-1), dict(flags=0x101), dict(flags=0x120), dict(flags=0x100, batch_start_delay_ms=-1), dict(flags=4, scale_interval_ms=0),
    dict(flags=0x20, scale_interval_ms=0), dict(flags=0x20, autoscale_f_milli=-1), dict(flags=0x20, autoscale_f_milli=100_001),
    dict(flags=0x20, scaling_buffer_hosts=-1), dict(flags=0x20, scaling_buffer_hosts=1025), dict(flags=0x24, min_hosts=-1),
    dict(flags=4, scale_in_idle_pct=101), dict(retry_interval_ms=2_000_000_000, max_retries=15),
    dict(flags=0x3000), dict(flags=0x10000)])
def test_create_rejects_bad_config(lib, bad):
    # no replays, so null arrays are fine and only the parameters can be at fault
    assert _create(lib, _cfg(**bad), n_replays=0) == replay.E_ARG
    assert _create(lib, _cfg(**bad)) == replay.E_ARG


def test_create_accepts_the_base_config_as_far_as_the_host_checks_go(lib):
    # the same call with nothing wrong gets past the parameter checks: it fails only for want of a
    # device (here), or succeeds (on a GPU machine)
    c = replay.make_config(_cfg(), 0, 1)
    ins = replay.NbosInputs()
    h = C.c_void_p()
    rc = lib.nbos_replay_create(C.byref(c), C.byref(ins), None, C.byref(h))
    assert rc in (replay.E_HIP, 0)
    if rc == 0:
        lib.nbos_replay_destroy(h)


@pytest.mark.parametrize("flags", [4, 0x20, 0x24])
def test_create_rejects_a_scaling_period_that_overflows_the_clock(lib, flags):
    # the auto-scaler's next period is scheduled one interval past the last instant of a replay: an
    # interval that takes that beyond 2^31 - 1 ms together with the longest cell is refused outright
    # (shorter ones shrink the time range a trace may use, checked against the trace on the device)
    day = 86_400_000
    assert _create(lib, _cfg(flags=flags, scale_interval_ms=2**31 - 1 - day), n_replays=0) == replay.E_ARG
    assert _create(lib, _cfg(flags=flags, scale_interval_ms=2**31 - 1), n_replays=0) == replay.E_ARG
    assert _create(lib, _cfg(flags=flags, scale_interval_ms=2**30), n_replays=0) in (replay.E_HIP, 0)
    # without a periodic rule the field is ignored
    assert _create(lib, _cfg(flags=1, scale_interval_ms=2**31 - 1), n_replays=0) in (replay.E_HIP, 0)


def test_create_rejects_null_and_size(lib):
    assert _create(lib, _cfg(), inputs=False) == replay.E_ARG
    assert _create(lib, _cfg(), out=False) == replay.E_ARG
    assert _create(lib, _cfg(), struct_size=12) == replay.E_ARG
    assert _create(lib, _cfg(), n_replays=-1) == replay.E_ARG
    assert _create(lib, _cfg(), n_replays=1, n_traces=0) == replay.E_ARG
    assert _create(lib, _cfg()) == replay.E_ARG                       # null arrays with n_replays > 0
    assert _create(lib, _cfg(hosts_initial=4, hosts_max=1025)) == replay.E_LIMIT


def test_null_handle_calls(lib):
    assert lib.nbos_replay_run(None) == replay.E_ARG
    assert lib.nbos_replay_stats(None, 0, 0, None) == replay.E_ARG
    assert lib.nbos_replay_decisions(None, 0, None, 0) == replay.E_ARG
    assert lib.nbos_replay_last_kernel_ms(None, None) == replay.E_ARG
    assert lib.nbos_replay_launch_info(None, None, None, None) == replay.E_ARG
    lib.nbos_replay_destroy(None)


def test_decision_codes_decode_to_their_fields():
    from helpers import code_of
    from paper_2503_20591_amd import replay
    # code_of(time, outcome, session, slot, host) builds codes the way the hand-worked traces list them
    d = replay.decode_decision(code_of(123456, 5, 4321, 2, 777))
    assert d == {"time_ms": 123456, "session": 4321, "outcome": 5, "name": "MIGRATE", "slot": 2, "host": 777}
    names = {int(m.group(2)): m.group(1) for m in re.finditer(r"#define NBOS_D_(\w+)\s+(\d+)", open(os.path.join(ROOT, "include", "nbos.h")).read())}
    assert names == replay.DECISION_NAMES
