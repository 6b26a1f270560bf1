"""GPU parity: the HIP replay (through the C ABI) against the CPU oracle, bit for bit.

All outputs are integers, so the bar is exact equality of every field of the result record,
including the digest of the decision sequence; where the decision log is on, the full sequence
of decision codes is compared too.
"""
import os

import numpy as np
import pytest

from helpers import GOLDEN, code_of, digest_of, events_to_arrays, load_golden
from paper_2503_20591_amd import tracegen as tg

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_20591_amd import replay
    replay.load()          # fails loudly if libnbos.so has not been built
    return replay


def gpu_run(rp, batch, log=False, in_lds=False, generic=False, rounds=None, one_wave=False):
    dev = rp.upload(batch)
    h = rp.Replay(batch.config, dev, decision_log=log, hosts_in_lds=in_lds, generic_kernel=generic, rounds=rounds,
                  one_wave=one_wave)
    h.run()
    st = h.stats()
    logs = [h.decisions(r) for r in range(batch.n_replays)] if log else None
    h.close()
    return st, logs


def as_batch(b, delay, scale_out):
    b.config.update(flags=tg.F_BATCH_MODE | (tg.F_SCALE_OUT if scale_out else 0), batch_start_delay_ms=delay)
    if not scale_out:
        b.config["hosts_max"] = b.config["hosts_initial"]
    return b


def first_diff(a, b, orc):
    for i, (x, y) in enumerate(zip(a, b)):
        if int(x) != int(y):
            return f"decision {i}: gpu {orc.decode(x)} oracle {orc.decode(y)}"
    return f"lengths {len(a)} vs {len(b)}"


def assert_same(rp, orc, batch, st, logs=None, replays=None, check=False):
    idx = range(batch.n_replays) if replays is None else replays
    for r in idx:
        t = int(batch.trace_of_replay[r])
        a, b = int(batch.ev_offset[t]), int(batch.ev_offset[t + 1])
        sa, sb = int(batch.sess_offset[t]), int(batch.sess_offset[t + 1])
        want = orc.replay(batch.config, batch.ev_time[a:b], batch.ev_dur[a:b], batch.ev_sk[a:b],
                          batch.sess_gpus[sa:sb], int(batch.cap_milli[r]), check=check, want_log=logs is not None)
        got = rp.stats_to_dict(st[r])
        assert got["status"] == 0, (batch.name, r, got["status"])
        if logs is not None and [int(x) for x in logs[r]] != [int(x) for x in want["log"]]:
            raise AssertionError(f"{batch.name} replay {r}: {first_diff(logs[r], want['log'], orc)}")
        for k in orc.RESULT_FIELDS:
            assert got[k] == want[k], (batch.name, r, k, got[k], want[k])


def assert_same_all(rp, orc, batch, st, threads=16):
    """Every replay of the batch against the oracle (the oracle's replays spread over host threads)."""
    want = orc.replay_batch(batch, threads=threads)
    assert len(want) == batch.n_replays == len(st)
    assert (st["status"] == 0).all(), batch.name
    for k in orc.RESULT_FIELDS:
        w = np.array([x[k] for x in want], dtype=np.uint64 if k == "digest" else np.int64)
        g = st[k].astype(w.dtype)
        if not np.array_equal(g, w):
            r = int(np.argwhere((g != w).reshape(len(st), -1).any(axis=1))[0, 0])
            raise AssertionError((batch.name, r, k, g[r].tolist(), w[r].tolist()))


# ---- hand-worked traces straight through the GPU ---------------------------------------------------

@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
@pytest.mark.parametrize("name", sorted(f for f in os.listdir(GOLDEN) if f.startswith("hand_")))
def test_hand_worked_gpu(rp, name, in_lds):
    g = load_golden(name)
    t, d, sk = events_to_arrays(g["events"])
    b = tg._pack(g["config"], [(t, d, sk, np.asarray(g["sess_gpus"], np.uint8))], [0], [g["cap_milli"]], name)
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    got = rp.stats_to_dict(st[0])
    for k, v in g["expect"].items():
        assert got[k] == v, (name, k, got[k], v)
    codes = [code_of(*x) for x in g["decisions"]]
    assert [int(x) for x in logs[0]] == codes
    assert got["digest"] == digest_of(codes)


# ---- randomized small clusters: every flag combination, odd delays, END events, shared traces -----

@pytest.mark.parametrize("seed", range(120))
def test_random_cases(rp, oracle, seed):
    b = tg.random_case(seed)
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs, check=True)


@pytest.mark.parametrize("seed", range(0, 120, 3))
def test_random_cases_hosts_in_lds(rp, oracle, seed):
    # the any-size kernel on the same cases (it is chosen by itself only above 64 hosts)
    b = tg.random_case(seed)
    st, logs = gpu_run(rp, b, log=True, in_lds=True)
    assert_same(rp, oracle, b, st, logs)


# ---- periodic auto-scaler (Section 3.4.2) and dynamic subscription-ratio limit (Section 3.4.1) -----

@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
@pytest.mark.parametrize("seed", range(60))
def test_policy_flag_cases(rp, oracle, seed, in_lds):
    b = tg.random_case(seed, policy_flags=True)
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs, check=not in_lds)


@pytest.mark.parametrize("f_milli,buf,min_hosts", [(1050, 200, 100), (4000, 8, 300)])
def test_autoscaler_on_a_large_cluster(rp, oracle, f_milli, buf, min_hosts):
    # the diurnal 512-host workload under the periodic auto-scaler (the paper's f = 1.05 with a large
    # buffer, and a more aggressive f with a small one), releases allowed, plus the dynamic limit:
    # hosts come and go all day
    b = tg.workload("c4", n_replays=2)
    b.config.update(flags=tg.F_MIGRATE | tg.F_SCALE_OUT | tg.F_SCALE_IN | tg.F_AUTOSCALE | tg.F_DYNAMIC_SR,
                    autoscale_f_milli=f_milli, scaling_buffer_hosts=buf, min_hosts=min_hosts)
    b.cap_milli = np.asarray([2000, 700], np.int32)
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)
    assert st["scale_in_hosts"].min() > 0
    auto = [sum(1 for c in lg if oracle.decode(c)["outcome"] == oracle.D_SCALE_AUTO) for lg in logs]
    assert max(auto) > 0


@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
def test_dynamic_limit_where_it_can_and_cannot_differ(rp, oracle, in_lds):
    # Section 3.4.1's dynamic limit equals the replay's cap when the cap admits any request on an empty host
    # and the cluster always has more hosts than a request has GPUs (the kernels then keep their fixed-cap
    # bounds); one host or one GPU of room less and it is worked out at every test. Both sides of that line,
    # on a loaded cluster that grows, shrinks and migrates: G = 4, 4 or 5 hosts at the start and as the floor
    # of the periodic release, caps that leave room for 3 or 4 subscribed GPUs per host.
    G = 4
    caps = [84, 167, 250, 333, 334, 1000]         # floor(cap * G * 3 / 1000) = 1, 2, 3, 3, 4, 12
    bites = 0
    for seed, (h0, min_hosts, hmax) in enumerate([(4, 4, 12), (5, 4, 12), (5, 5, 20), (6, 5, 30), (3, 3, 30), (5, 5, 9)]):
        tr = tg.make_trace(1000 + seed, 80, 2000, ramp_ms=120_000,
                           gpus=lambda r, n: np.minimum(tg.gpus_uniform(r, n), G).astype(np.uint8),
                           gap=lambda r, s: tg.exp_ms(r, 8.0, s), dur=lambda r, s: tg.lognormal_ms(r, 20.0, 1.0, s),
                           with_end=True)
        cfg = tg._base_config(hosts_initial=h0, hosts_max=hmax, gpus_per_host=G,
                              flags=tg.F_MIGRATE | tg.F_SCALE_OUT | tg.F_SCALE_IN | tg.F_DYNAMIC_SR,
                              migration_delay_ms=500, boot_delay_ms=2000, retry_interval_ms=3000,
                              max_retries=4, scale_interval_ms=7000, scale_in_idle_pct=10, min_hosts=min_hosts)
        b = tg._pack(cfg, [tr], [0] * len(caps), caps, f"dynlim{seed}")
        st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
        assert_same(rp, oracle, b, st, logs, check=not in_lds)
        # the same replays under the fixed cap alone: where does the dynamic limit change the outcome?
        fixed = tg._pack(dict(cfg, flags=cfg["flags"] & ~tg.F_DYNAMIC_SR), [tr], [0] * len(caps), caps, "fixed")
        for k, res in enumerate(oracle.replay_batch(fixed)):
            differs = int(res["digest"]) != int(st["digest"][k])
            bites += differs
            if caps[k] * G * 3 // 1000 >= G and min(h0, min_hosts) > G:
                assert not differs
    assert bites >= 8


def test_named_workload_c4a_autoscaler_only(rp, oracle):
    b = tg.workload("c4a", n_replays=2)
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)
    auto = [sum(1 for c in lg if oracle.decode(c)["outcome"] == oracle.D_SCALE_AUTO) for lg in logs]
    assert min(auto) > 0 and st["scale_in_hosts"].min() > 0


# ---- billing post-pass (section "Monetary Cost") ---------------------------------------------------------------

@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
def test_billing_matches_oracle(rp, oracle, in_lds):
    for seed, price, mk, sb in [(3, 10_000_000, 115, 125), (8, 1_000_000_000, 1000, 1000), (21, 1, 100, 0),
                                (40, 32_770_000, 115, 125), (77, 0, 115, 125)]:
        b = tg.random_case(seed, n_replays=5)
        dev = rp.upload(b)
        h = rp.Replay(b.config, dev, hosts_in_lds=in_lds)
        h.run()
        bills = h.billing(price, mk, sb)
        part = h.billing(price, mk, sb, first=2, count=2)
        h.close()
        want = oracle.replay_batch(b)
        for r in range(b.n_replays):
            exp = oracle.billing(want[r], b.config["gpus_per_host"], price, mk, sb)
            for k, v in exp.items():
                assert int(bills[k][r]) == v, (seed, r, k)
        assert (part == bills[2:4]).all()


def test_billing_printed_example_gpu(rp):
    # Section "Monetary Cost": $10 per 8-GPU host-hour, x1.15, standby 12.5 %: $5.75 for an hour on 4 GPUs,
    # $1.4375 (printed $1.44) per standby replica-hour
    HOUR = 3_600_000
    t, d, sk = events_to_arrays([[0, 0, 0, 0], [0, 1, 0, HOUR], [2 * HOUR, 2, 0, 0]])
    cfg = tg._base_config(hosts_initial=3, hosts_max=3, flags=0)
    b = tg._pack(cfg, [(t, d, sk, np.asarray([4], np.uint8))], [0], [1000], "billing")
    dev = rp.upload(b)
    h = rp.Replay(b.config, dev)
    h.run()
    bill = h.billing(10_000_000)[0]
    st = h.stats()[0]
    h.close()
    assert int(st["replica_ms"]) == 6 * HOUR
    assert int(bill["usage_revenue"]) == 5_750_000
    assert int(bill["standby_revenue"]) == 5 * 1_437_500
    assert int(bill["provider_cost"]) == 60_000_000
    assert int(bill["reservation_revenue"]) == 11_500_000


def test_billing_of_the_batch_baseline(rp, oracle):
    # no replicas there: no standby charge, usage and provider cost as usual
    b = as_batch(tg.random_case(5, n_replays=3), delay=500, scale_out=False)
    dev = rp.upload(b)
    h = rp.Replay(b.config, dev)
    h.run()
    bills = h.billing(10_000_000)
    h.close()
    want = oracle.replay_batch(b)
    for r in range(b.n_replays):
        exp = oracle.billing(want[r], b.config["gpus_per_host"], 10_000_000)
        assert exp["standby_revenue"] == 0
        for k, v in exp.items():
            assert int(bills[k][r]) == v, (r, k)


def test_billing_rejects_bad_arguments(rp):
    b = tg.random_case(1, n_replays=2)
    dev = rp.upload(b)
    h = rp.Replay(b.config, dev)
    with pytest.raises(rp.NbosError) as e:
        h.billing(10_000_000)                      # never run
    assert e.value.code == rp.E_STATE
    h.run()
    for kw in (dict(price_micro_per_host_hour=-1), dict(price_micro_per_host_hour=10**9 + 1),
               dict(price_micro_per_host_hour=1, markup_pct=1001), dict(price_micro_per_host_hour=1, standby_permille=-1),
               dict(price_micro_per_host_hour=1, first=1, count=2)):
        with pytest.raises(rp.NbosError) as e:
            h.billing(**kw)
        assert e.value.code == rp.E_ARG
    h.close()


@pytest.mark.parametrize("generic", [False, True], ids=["instances", "generic"])
def test_generic_and_specialised_register_kernels(rp, oracle, generic):
    # flag sets 0, MIGRATE and MIGRATE|SCALE_OUT have kernels of their own for small batches; large
    # batches run the generic kernel. Both must give the oracle's results on the same cases.
    done = set()
    for seed in range(200):
        b = tg.random_case(seed, n_replays=3)
        f = b.config["flags"]
        if f not in (0, 1, 3) or b.config["hosts_max"] > 64 or (f, (b.config["hosts_max"] + 7) // 8) in done:
            continue
        done.add((f, (b.config["hosts_max"] + 7) // 8))
        st, logs = gpu_run(rp, b, log=True, generic=generic)
        assert_same(rp, oracle, b, st, logs)
    assert len(done) >= 6
    # the any-size kernel has instances for MIGRATE and MIGRATE|SCALE_OUT|SCALE_IN
    seen = set()
    for seed in range(200):
        b = tg.random_case(seed, n_replays=3)
        if b.config["flags"] in (1, 7) and b.config["flags"] not in seen:
            seen.add(b.config["flags"])
            st, logs = gpu_run(rp, b, log=True, in_lds=True, generic=generic)
            assert_same(rp, oracle, b, st, logs)
    assert seen == {1, 7}
    for name, n in (("c2", 3), ("c5", 8)):
        b = tg.workload(name, n_replays=n)
        st, _ = gpu_run(rp, b, generic=generic)
        assert_same(rp, oracle, b, st)


# ---- Batch baseline (the paper's "Baselines" section) ------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(60))
def test_batch_mode_random_cases(rp, oracle, seed):
    b = tg.random_case(seed)
    as_batch(b, delay=[0, 1, 40, 15_000][seed % 4], scale_out=bool(b.config["flags"] & tg.F_SCALE_OUT))
    if seed % 5 == 0:                      # room to grow
        b.config["hosts_max"] = b.config["hosts_initial"] + 7
        b.config["flags"] |= tg.F_SCALE_OUT
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs, check=True)


@pytest.mark.parametrize("name,n,hosts", [("c2", 4, 30), ("c2", 2, 6), ("c5", 8, 16), ("c4", 1, 512), ("c4", 1, 96)])
def test_batch_mode_named_workloads(rp, oracle, name, n, hosts):
    # the NotebookOS workloads replayed under the Batch baseline, also on far fewer hosts (long queues)
    b = tg.workload(name, n_replays=n)
    as_batch(b, delay=20_000, scale_out=False)
    b.config["hosts_initial"] = b.config["hosts_max"] = hosts
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)
    assert (st["cells_started"] + st["cells_dropped_busy"] == st["cells_total"]).all()


@pytest.mark.parametrize("h0,hmax,name", [(60, 70, "c2"), (64, 66, "c2"), (63, 129, "c5"), (120, 200, "c3")])
def test_batch_mode_grows_across_chunks_of_hosts(rp, oracle, h0, hmax, name):
    # the Batch kernel keeps minima per chunk of 64 hosts on clusters of more than 64: hosts are added on
    # demand into a chunk that was empty, into one that is partly on, and the last chunk is ragged
    b = tg.workload(name, n_replays=3)
    as_batch(b, delay=5_000, scale_out=True)
    b.config.update(hosts_initial=h0, hosts_max=hmax, boot_delay_ms=30_000)
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs, check=True)
    assert st["scale_out_hosts"].max() > 0 and st["cells_queued"].max() > 0


def test_batch_mode_time_range(rp, oracle):
    # 30 one-day jobs on a single host: the 25th would end beyond 2^31 - 1 ms. Both sides call the
    # replay invalid (the oracle returns its input error, the kernel sets the replay's status).
    n = 30
    t, d, sk = events_to_arrays([[i, 1, i, 86_400_000] for i in range(n)])
    cfg = tg._base_config(hosts_initial=1, hosts_max=1, flags=tg.F_BATCH_MODE)
    b = tg._pack(cfg, [(t, d, sk, np.full(n, 8, np.uint8))], [0, 0], [1000, 1000], "overflow")
    with pytest.raises(ValueError) as e:
        oracle.replay_batch(b)
    assert e.value.args[1] == -2
    st, _ = gpu_run(rp, b)
    assert (st["status"] == rp.E_RANGE).all()
    # one job fewer than the limit allows is fine
    n = 24
    t, d, sk = events_to_arrays([[i, 1, i, 86_400_000] for i in range(n)])
    b = tg._pack(cfg, [(t, d, sk, np.full(n, 8, np.uint8))], [0], [1000], "no-overflow")
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)


def test_batch_mode_rejects_other_policy_flags(rp):
    b = tg.random_case(2)
    dev = rp.upload(b)
    for f in (tg.F_BATCH_MODE | tg.F_MIGRATE, tg.F_BATCH_MODE | tg.F_SCALE_IN, tg.F_BATCH_MODE | tg.F_AUTOSCALE):
        cfg = dict(b.config, flags=f)
        with pytest.raises(rp.NbosError) as e:
            rp.Replay(cfg, dev)
        assert e.value.code == rp.E_ARG


# ---- closed-loop reading of the traces (the section "Interactive Deep Learning Training": users think between the cells they submit) ------

def as_closed(b):
    b.config["flags"] = (b.config["flags"] & ~(tg.F_SCALE_IN | tg.F_AUTOSCALE)) | tg.F_CLOSED_LOOP
    return b


@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
@pytest.mark.parametrize("seed", range(60))
def test_closed_loop_random_cases(rp, oracle, seed, in_lds):
    # clusters of up to 64 hosts run on the register kernel's closed loop unless the other one is asked for
    b = as_closed(tg.random_case(seed))
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs, check=not in_lds)


@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
@pytest.mark.parametrize("seed", range(30))
def test_closed_loop_policy_flag_cases(rp, oracle, seed, in_lds):
    # with the dynamic limit, the sticky executor and the pre-warmed containers
    b = as_closed(tg.random_case(seed, policy_flags=True))
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs, check=not in_lds)


@pytest.mark.parametrize("name,n,in_lds", [("c2l", 6, False), ("c2l", 6, True), ("c4l", 2, False)])
def test_closed_loop_named_workloads(rp, oracle, name, n, in_lds):
    b = tg.workload(name, n_replays=n)
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs)
    assert (st["cells_dropped_busy"] == 0).all()          # a session never submits while its cell runs
    assert (st["cells_total"] == st["cells_started"] + st["cells_aborted"]).all()


@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
@pytest.mark.parametrize("name,n", [("c3", 4), ("c5", 16), ("c1", 1)])
def test_closed_loop_on_the_other_traces(rp, oracle, name, n, in_lds):
    # 1,000 sessions on 64 hosts: nearly every session's timer waits in its record, not in the
    # 64 sorted slots (refill takes several at once, pushes evict the latest)
    b = as_closed(tg.workload(name, n_replays=n))
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs, check=name != "c3" and not in_lds)


@pytest.mark.parametrize("seed", range(0, 60, 2))
def test_closed_loop_random_cases_with_forced_rounds(rp, oracle, seed):
    # small clusters run without the event-parallel rounds by default: here with them
    b = as_closed(tg.random_case(seed, policy_flags=seed % 4 == 0))
    st, logs = gpu_run(rp, b, log=True, in_lds=True, rounds=True)
    assert_same(rp, oracle, b, st, logs, check=True)


def test_closed_loop_named_workloads_with_forced_rounds(rp, oracle):
    for name, n in (("c2l", 3), ("c3", 2), ("c5", 8)):
        b = as_closed(tg.workload(name, n_replays=n))
        st, logs = gpu_run(rp, b, log=True, in_lds=True, rounds=True)
        assert_same(rp, oracle, b, st, logs)
    # all sessions' cells due at the same instants, again and again
    test_closed_loop_many_timers_at_one_instant(rp, oracle, True, rounds=True)


def test_closed_loop_without_the_parallel_rounds(rp, oracle):
    # the same replays with every timer fired one by one
    for name, n in (("c3", 2), ("c4l", 1)):
        b = as_closed(tg.workload(name, n_replays=n))
        st, logs = gpu_run(rp, b, log=True, rounds=False)
        assert_same(rp, oracle, b, st, logs)


def test_closed_loop_without_log_full_batch(rp, oracle):
    # the whole c2l batch in the launch shape the benchmark uses, every replay against the oracle
    b = tg.workload("c2l", workers=8)
    st, _ = gpu_run(rp, b)
    assert (st["status"] == 0).all()
    assert_same_all(rp, oracle, b, st)
    assert (st["cells_total"] == st["cells_started"] + st["cells_aborted"]).all()
    # the same handle run twice more: nothing of a run (cursors, waiting timers) leaks into the next
    h = rp.Replay(b.config, rp.upload(b))
    h.run(); h.run()
    st2 = h.stats()
    h.close()
    assert st2.tobytes() == st.tobytes()


@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
def test_closed_loop_many_timers_at_one_instant(rp, oracle, in_lds, rounds=None):
    # 300 sessions placed at time 0 whose first cells are all due at the same millisecond, and again
    # later: far more than 64 timers for one instant wait outside the sorted slots, so they are
    # taken one by one in (kind, session) order; mixed with retries of queued cells
    n = 300
    rng = np.random.default_rng(4)
    ev = [[0, 0, s, 0] for s in range(n)]
    ev += [[5000, 1, s, 2000] for s in range(n)]                 # think 5000 after the placement
    ev += [[9000, 1, s, 1000 + 1000 * (s % 3)] for s in range(n)]   # think 2000 after the first cell
    ev += [[20000 + s, 2, s, 0] for s in range(0, n, 2)]
    cfg = dict(BASE, hosts_initial=6, hosts_max=6, flags=tg.F_MIGRATE | tg.F_CLOSED_LOOP, migration_delay_ms=300,
               retry_interval_ms=1000, max_retries=3)
    gp = rng.choice([1, 2, 4], n)
    b = _tiny(cfg, ev, gp, [100000, 6000])
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds, rounds=rounds)
    assert_same(rp, oracle, b, st, logs, check=True)
    assert st["cells_queued"].max() > 64


@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
def test_closed_loop_time_range(rp, oracle, in_lds):
    # Three sessions keep all three hosts busy for a day, twice; the fourth session's first two cells
    # are given up after a minute each, so its third cell, nominally at the latest time a trace may
    # hold, comes two minutes late: with a one-day duration it would end beyond 2^31 - 1 ms. Both
    # sides call the replay invalid; 59,998 ms less and it ends at 2^31 - 2 and is fine.
    day = 86_400_000
    cfg = tg._base_config(hosts_initial=3, hosts_max=3, gpus_per_host=8, flags=tg.F_CLOSED_LOOP,
                          migration_delay_ms=0, boot_delay_ms=0, retry_interval_ms=10_000, max_retries=6)
    t_limit = 2**31 - 2 - (day + 6 * 10_000)

    def batch(d3):
        ev = [[0, 0, s, 0] for s in range(4)]
        ev += [[10, 1, s, day] for s in range(3)] + [[20, 1, 3, 1]]
        ev += [[10 + day + 5, 1, s, day] for s in range(3)] + [[10 + day + 100, 1, 3, 1]]
        ev += [[t_limit, 1, 3, d3]]
        return _tiny(cfg, ev, [8, 8, 8, 8], [100000])

    for d3 in (day, day - 59_997):
        b = batch(d3)
        with pytest.raises(ValueError) as e:
            oracle.replay(b.config, b.ev_time, b.ev_dur, b.ev_sk, b.sess_gpus, 100000)
        assert e.value.args[1] == -2
        st, _ = gpu_run(rp, b, in_lds=in_lds)
        assert (st["status"] == rp.E_RANGE).all()
    b = batch(day - 59_998)
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs, check=True)
    assert st["t_end_ms"][0] == 2**31 - 2


def test_closed_loop_rejects_periodic_scaling_and_batch(rp):
    b = tg.random_case(2)
    dev = rp.upload(b)
    for f in (tg.F_SCALE_IN, tg.F_AUTOSCALE | tg.F_SCALE_IN, tg.F_BATCH_MODE):
        cfg = dict(b.config, flags=tg.F_CLOSED_LOOP | f)
        with pytest.raises(rp.NbosError) as e:
            rp.Replay(cfg, dev)
        assert e.value.code == rp.E_ARG


def test_random_cases_without_log(rp, oracle):
    for seed in range(120, 150):
        b = tg.random_case(seed, n_replays=6)
        st, _ = gpu_run(rp, b)
        assert_same(rp, oracle, b, st)


# ---- the five named workloads at reduced replay counts (full per-replay size) ----------------------

@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
@pytest.mark.parametrize("name,n", [("c1", 1), ("c2", 6), ("c3", 4), ("c5", 24)])
def test_named_workloads(rp, oracle, name, n, in_lds):
    b = tg.workload(name, n_replays=n)
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs)


@pytest.mark.parametrize("one_wave", [False, True], ids=["helper-waves", "one-wave"])
def test_named_workload_c4_many_hosts(rp, oracle, one_wave):
    # 512 -> 768 hosts: twelve chunks of 64 hosts per scan (shared by four waves, or all in one), scale-out,
    # scale-in, END events
    b = tg.workload("c4", n_replays=2)
    dev = rp.upload(b)
    h = rp.Replay(b.config, dev, decision_log=True, one_wave=one_wave)
    assert h.launch_info()["threads_per_group"] == (64 if one_wave else 256)
    h.close()
    st, logs = gpu_run(rp, b, log=True, one_wave=one_wave)
    assert_same(rp, oracle, b, st, logs)
    assert st["scale_out_hosts"].min() > 0


@pytest.mark.parametrize("name,n", [("c4a", 2), ("c4l", 2)])
def test_large_clusters_without_helper_waves(rp, oracle, name, n):
    # the auto-scaler workload and the closed loop on one wave per replay (the default there is four)
    b = tg.workload(name, n_replays=n)
    st, logs = gpu_run(rp, b, log=True, one_wave=True)
    assert_same(rp, oracle, b, st, logs)


@pytest.mark.parametrize("hosts", [192, 193, 256, 320, 1000, 1024])
def test_helper_waves_on_ragged_host_counts(rp, oracle, hosts):
    # 193 hosts and more run with helper waves: host counts that leave some waves without a chunk, or with a
    # partly filled one; migration, scale-out from a smaller start, periodic scale-in, END events
    cfg = tg.workload("c4", n_replays=1).config
    b = tg.workload("c4" if hosts <= 768 else "c3", n_replays=1)      # (8,000 sessions fit beside 768 hosts at most)
    b.config = dict(cfg, hosts_initial=max(hosts - 40, 1), hosts_max=hosts, min_hosts=hosts // 2)
    b.cap_milli[:] = 400                      # a low cap: placements run out of hosts and add some
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)


# ---- the benchmark configuration at full size: sampled replays + properties that hold for all -----

def test_full_size_bench_config(rp, oracle):
    # the largest named workload, which the benchmark times: all 256 replays against the oracle
    b = tg.workload("c4", workers=16)
    assert b.n_replays == 256 and b.config["hosts_initial"] == 512 and b.config["hosts_max"] == 768
    st, _ = gpu_run(rp, b)
    assert_same_all(rp, oracle, b, st)
    assert (st["cells_total"] == 500_000).all()
    assert (st["cells_total"] == st["cells_started"] + st["cells_aborted"] + st["cells_dropped_busy"]
            + st["cells_dropped_unplaced"]).all()
    assert (st["delay_hist"].sum(axis=1) == st["cells_started"]).all()
    assert (st["sessions_placed"] + st["sessions_rejected"] == 8000).all()
    assert (st["gpu_ms_committed"] - st["gpu_ms_executed"] >= 0).all()
    # a second run of the same handle recomputes the same results
    dev = rp.upload(b)
    h = rp.Replay(b.config, dev)
    h.run(); h.run()
    st2 = h.stats()
    h.close()
    assert st2.tobytes() == st.tobytes()


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c5", "c4a", "c2b", "c4b", "c2l", "c4l"])
def test_full_size_other_configs(rp, oracle, name):
    # the other named workloads with all their replays, in the launch shape the benchmark times (c2: one
    # wave per SIMD, c3: 16 workgroups per compute unit resident, c5: 64 per compute unit in several
    # rounds, the kernel flavour chosen for that shape): every replay against the oracle
    b = tg.workload(name, workers=16)
    st, _ = gpu_run(rp, b)
    assert_same_all(rp, oracle, b, st)
    assert (st["cells_total"] == st["cells_started"] + st["cells_aborted"] + st["cells_dropped_busy"]
            + st["cells_dropped_unplaced"]).all()
    assert (st["delay_hist"].sum(axis=1) == st["cells_started"]).all()
    assert (st["gpu_ms_committed"] >= st["gpu_ms_executed"]).all()
    if name == "c2":
        assert (st["gpu_ms_provisioned"] == 30 * 8 * st["t_end_ms"].astype(np.int64)).all()


# ---- edge cases ---------------------------------------------------------------------------------------

def _tiny(cfg, events, gpus, caps, tor=None):
    t, d, sk = events_to_arrays(events)
    return tg._pack(cfg, [(t, d, sk, np.asarray(gpus, np.uint8))], tor if tor is not None else [0] * len(caps), caps, "tiny")


BASE = dict(hosts_initial=3, hosts_max=3, gpus_per_host=8, flags=0, migration_delay_ms=0, boot_delay_ms=0,
            retry_interval_ms=100, max_retries=2, scale_interval_ms=1000, scale_in_idle_pct=0, min_hosts=0)


def test_empty_trace_and_no_replays(rp, oracle):
    b = _tiny(BASE, [], [1], [2000])
    st, _ = gpu_run(rp, b)
    assert_same(rp, oracle, b, st)
    assert st["t_end_ms"][0] == 0 and st["digest"][0] == 0xCBF29CE484222325
    b0 = _tiny(BASE, [[0, 0, 0, 0]], [1], [])
    dev = rp.upload(b0)
    h = rp.Replay(b0.config, dev)
    h.run()
    assert h.stats().shape == (0,)
    h.close()


def test_ragged_tail_sizes(rp, oracle):
    # event counts around the 64-event tile: 1, 63, 64, 65, 127, 128, 129
    traces = []
    for n in (1, 63, 64, 65, 127, 128, 129):
        ev = [[0, 0, 0, 0]] + [[10 * i, 1, 0, 7] for i in range(1, n)]
        t, d, sk = events_to_arrays(ev)
        traces.append((t, d, sk, np.asarray([2], np.uint8)))
    b = tg._pack(BASE, traces, list(range(len(traces))), [2000] * len(traces), "ragged")
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)


def test_max_hosts_and_single_gpu(rp, oracle):
    cfg = dict(BASE, hosts_initial=1000, hosts_max=1024, gpus_per_host=1, flags=7, boot_delay_ms=50,
               migration_delay_ms=20, scale_interval_ms=500, scale_in_idle_pct=5, min_hosts=900)
    rng = np.random.default_rng(1)
    n = 600
    ev = [[i, 0, i, 0] for i in range(n)]
    tcur = n
    for i in range(3000):
        tcur += int(rng.integers(0, 3))
        ev.append([tcur, 1, int(rng.integers(0, n)), int(rng.integers(1, 400))])
    ev += [[tcur + 5, 2, i, 0] for i in range(0, n, 2)]
    b = _tiny(cfg, ev, [1] * n, [334, 1000])
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)


@pytest.mark.parametrize("in_lds", [False, True], ids=["regs", "lds"])
def test_many_pending_timers(rp, oracle, in_lds):
    # far more than 64 timers pending at once (retries of queued cells and deferred ENDs), so the
    # timers that do not fit the 64 sorted slots are exercised: refill, eviction, END while queued
    rng = np.random.default_rng(9)
    n = 400
    cfg = dict(BASE, hosts_initial=5, hosts_max=5, gpus_per_host=8, flags=1, migration_delay_ms=700,
               retry_interval_ms=3000, max_retries=6)
    ev = [[i, 0, i, 0] for i in range(n)]
    t = n
    for rnd in range(6):
        for s in rng.permutation(n):
            t += int(rng.integers(0, 40))
            ev.append([t, 1, int(s), int(rng.integers(2000, 60000))])
            if rng.random() < 0.15:
                ev.append([t + 1, 2, int(s), 0]); t += 1
    gp = rng.choice([2, 4, 8], n)
    b = _tiny(cfg, ev, gp, [2000, 100000])
    st, logs = gpu_run(rp, b, log=True, in_lds=in_lds)
    assert_same(rp, oracle, b, st, logs, check=True)
    assert st["cells_queued"].max() > 500


@pytest.mark.parametrize("hosts", [70, 200])
def test_thousands_of_timers_pending_at_once(rp, oracle, hosts):
    # 8,000 sessions of 8 GPUs submit within eight seconds on a cluster that runs a few dozen cells at a time:
    # thousands of retry timers wait outside the 64 sorted ones at once (the any-size kernel keeps them in the
    # session records, so none can be turned away), are retried six times and given up; some sessions end
    # while queued. 70 hosts: one wave per replay; 200 hosts: with helper waves.
    n = 8000
    rng = np.random.default_rng(3)
    ev = [[s, 0, s, 0] for s in range(n)]
    ev += [[10_000 + s, 1, s, int(rng.integers(20_000, 200_000))] for s in range(n)]
    ev += [[30_000 + s, 2, s, 0] for s in range(0, n, 5)]
    ev.sort(key=lambda e: e[0])
    cfg = dict(BASE, hosts_initial=hosts, hosts_max=hosts, flags=tg.F_MIGRATE, migration_delay_ms=500,
               retry_interval_ms=10_000, max_retries=6)
    b = _tiny(cfg, ev, np.full(n, 8, np.uint8), [100000, 3000])
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)
    assert st["cells_queued"][0] > 6900 and (st["status"] == 0).all()   # the replay without a subscription cap


def test_results_do_not_depend_on_the_launch_order(rp):
    # the library hands the replays out longest first (events of the trace, then cap); every replay still
    # writes the records of its own index: a batch and the same batch with its replays shuffled give the
    # same records, shuffled
    import copy
    b = tg.workload("c5", n_replays=96)
    st, _ = gpu_run(rp, b)
    perm = np.random.default_rng(5).permutation(b.n_replays)
    bb = copy.copy(b)
    bb.cap_milli = b.cap_milli[perm].copy()
    bb.trace_of_replay = b.trace_of_replay[perm].copy()
    st2, _ = gpu_run(rp, bb)
    for name in st.dtype.names:
        assert (st2[name] == st[name][perm]).all(), name
    assert len(set(int(x) for x in st["digest"])) > 90          # (the replays do differ)


def test_time_near_int32_limit(rp, oracle):
    cfg = dict(BASE, flags=1, migration_delay_ms=15000, retry_interval_ms=10000, max_retries=6)
    t0 = 2**31 - 2 - 86_400_000 - 6 * 10000 - 15000
    ev = [[0, 0, 0, 0], [0, 0, 1, 0], [t0 - 5, 1, 0, 86_400_000], [t0, 1, 1, 86_400_000]]
    b = _tiny(cfg, ev, [8, 8], [2000])
    st, logs = gpu_run(rp, b, log=True)
    assert_same(rp, oracle, b, st, logs)


def test_create_rejects_bad_traces(rp):
    def rc(events, gpus, caps=(2000,), tor=None, cfg=BASE):
        b = _tiny(cfg, events, gpus, list(caps), tor)
        with pytest.raises(rp.NbosError) as e:
            rp.Replay(b.config, rp.upload(b))
        return e.value.code
    assert rc([[5, 0, 0, 0], [4, 1, 0, 1]], [1]) == rp.E_RANGE          # unsorted
    assert rc([[0, 1, 0, 0]], [1]) == rp.E_RANGE                        # duration 0
    assert rc([[0, 1, 1, 5]], [1]) == rp.E_RANGE                        # session out of range
    assert rc([[0, 3, 0, 5]], [1]) == rp.E_RANGE                        # kind out of range
    assert rc([[0, 0, 0, 0]], [9]) == rp.E_RANGE                        # g > G
    assert rc([[2_100_000_000, 0, 0, 0]], [1]) == rp.E_RANGE            # time overflow
    assert rc([[0, 0, 0, 0]], [1], caps=(0,)) == rp.E_RANGE             # cap out of range
    assert rc([[0, 0, 0, 0]], [1], tor=[1]) == rp.E_RANGE               # trace index out of range


def test_stats_before_run_is_an_error(rp):
    b = _tiny(BASE, [[0, 0, 0, 0]], [1], [2000])
    h = rp.Replay(b.config, rp.upload(b))
    with pytest.raises(rp.NbosError) as e:
        h.stats()
    assert e.value.code == rp.E_STATE
    with pytest.raises(rp.NbosError):
        h.decisions(0)
    h.close()


def test_runs_on_a_side_stream(rp, oracle):
    import torch
    b = tg.random_case(7)
    dev = rp.upload(b)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    h = rp.Replay(b.config, dev, stream=s)
    h.run()
    st = h.stats()
    assert h.last_kernel_ms() > 0
    h.close()
    assert_same(rp, oracle, b, st)
