"""The entry point that allocates nothing (nbos_replay_run_static) against create + run + stats.

Two calls in a row through the C ABI on one GPU, the second on a smaller input: the scratch array
inside the library is shared by all calls and keeps the last call's contents."""
import numpy as np
import pytest

from paper_2503_20591_amd import tracegen as tg

pytestmark = pytest.mark.gpu


def _both(rp, torch, batch):
    print("case", batch.name, batch.n_replays, flush=True)
    dev = rp.upload(batch)
    h = rp.Replay(batch.config, dev)
    h.run()
    want = h.stats()
    h.close()
    n_cap = int(np.diff(batch.sess_offset).max()) if batch.n_traces else 0
    out = torch.full((batch.n_replays * rp.STATS_DTYPE.itemsize,), 0xAB, dtype=torch.uint8, device="cuda:0")
    rp.run_static(batch.config, dev, n_cap, out)
    torch.cuda.synchronize()
    got = rp.stats_from_tensor(out, batch.n_replays)
    assert (want["status"] == 0).all()
    _same(rp, got, want, batch.name)
    return dev


def _same(rp, got, want, what):
    # field by field: the records have four bytes of padding that nobody writes
    for k in rp.STATS_DTYPE.names:
        assert np.array_equal(got[k], want[k]), (what, k)


def test_static_entry_point_matches_the_handle_path_twice():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_20591_amd import replay as rp
    rp.load()
    # first call: c2 traces (30 hosts, 400 sessions, migration; hundreds of queued cells per replay, so the
    # queued durations go through the scratch array), then a smaller and different batch (c5: scale-out)
    _both(rp, torch, tg.workload("c2", n_replays=96, workers=8))
    _both(rp, torch, tg.workload("c5", n_replays=40, workers=8))
    # many timers waiting outside the sorted registers at once: the scratch array is what holds their cells
    rng = np.random.default_rng(9)
    n = 400
    cfg = dict(hosts_initial=5, hosts_max=5, gpus_per_host=8, flags=1, migration_delay_ms=700, boot_delay_ms=0,
               retry_interval_ms=3000, max_retries=6, scale_interval_ms=1000, scale_in_idle_pct=0, min_hosts=0)
    ev = [[i, 0, i, 0] for i in range(n)]
    t = n
    for _ in range(4):
        for s in rng.permutation(n):
            t += int(rng.integers(0, 40))
            ev.append([t, 1, int(s), int(rng.integers(2000, 60000))])
    e = np.asarray(ev, dtype=np.int64)
    tr = (e[:, 0].astype(np.int32), e[:, 3].astype(np.int32), (e[:, 2] | (e[:, 1] << 24)).astype(np.int32),
          rng.choice([2, 4, 8], n).astype(np.uint8))
    _both(rp, torch, tg.pack(cfg, [tr], [0, 0, 0], [2000, 100000, 1000], "queued"))


def test_static_entry_point_refuses_what_it_cannot_hold():
    import torch
    from paper_2503_20591_amd import replay as rp
    rp.load()
    b = tg.workload("c5", n_replays=8)
    dev = rp.upload(b)
    out = torch.zeros(b.n_replays * rp.STATS_DTYPE.itemsize, dtype=torch.uint8, device="cuda:0")
    big = dict(b.config, hosts_initial=65, hosts_max=65)
    with pytest.raises(rp.NbosError) as e:
        rp.run_static(big, dev, 120, out)
    assert e.value.code == rp.E_LIMIT
    with pytest.raises(rp.NbosError) as e:
        rp.run_static(b.config, dev, 65536 * 16, out)            # beyond the session limit
    assert e.value.code == rp.E_ARG
    with pytest.raises(rp.NbosError) as e:
        rp.run_static(dict(b.config, flags=b.config["flags"] | tg.F_CLOSED_LOOP), dev, 120, out)
    assert e.value.code == rp.E_ARG
    # more sessions in a trace than the caller said: the records say so, nothing is touched out of bounds
    rp.run_static(b.config, dev, 100, out)
    torch.cuda.synchronize()
    st = rp.stats_from_tensor(out, b.n_replays)
    assert (st["status"] == rp.E_LIMIT).all() and (st["cells_total"] == 0).all()
    # invalid trace content: every record carries NBOS_E_RANGE
    bad = dict(dev)
    bad["cap_milli"] = torch.zeros_like(dev["cap_milli"])
    rp.run_static(b.config, bad, 120, out)
    torch.cuda.synchronize()
    st = rp.stats_from_tensor(out, b.n_replays)
    assert (st["status"] == rp.E_RANGE).all()
    # and a good call afterwards is not disturbed by what the refused ones left behind
    rp.run_static(b.config, dev, 120, out)
    torch.cuda.synchronize()
    st = rp.stats_from_tensor(out, b.n_replays)
    h = rp.Replay(b.config, dev)
    h.run()
    _same(rp, st, h.stats(), "after refusals")
    h.close()
