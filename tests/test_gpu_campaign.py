"""GPU parity on mid-size randomized cases: traces drawn with the recipes of the named workloads at
random sizes, replayed on random cluster shapes under every mode (open loop on both kernels, closed
loop, Batch baseline, auto-scaler, pre-warmed pool), with the event-parallel rounds left to the
library, forced on and forced off. Every field of every result record against the oracle."""
import numpy as np
import pytest

from paper_2503_20591_amd import tracegen as tg

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(seed)
    base = str(rng.choice(["c2", "c3", "c4", "c5"]))
    kw = tg.recipe(base)["kw"]
    n_sess, n_cells = int(rng.integers(50, 900)), int(rng.integers(2000, 40000))
    traces = [tg.make_trace(seed * 7 + i, n_sess, n_cells, **kw) for i in range(2)]
    h0 = int(rng.choice([3, 8, 20, 40, 64, 65, 100, 200, 400]))
    flags = int(rng.integers(0, 8)) | (tg.F_STICKY_EXECUTOR if rng.random() < 0.3 else 0) | \
        (tg.F_DYNAMIC_SR if rng.random() < 0.3 else 0)
    mode = str(rng.choice(["open", "open", "closed", "batch", "auto", "warm"]))
    cfg = tg.base_config(
        hosts_initial=h0, hosts_max=h0 + (int(rng.integers(0, 100)) if flags & tg.F_SCALE_OUT else 0),
        gpus_per_host=int(rng.choice([1, 2, 4, 8, 8])), flags=flags,
        migration_delay_ms=int(rng.choice([0, 500, 15000])), boot_delay_ms=int(rng.choice([0, 2000, 60000])),
        retry_interval_ms=int(rng.choice([700, 10000])), max_retries=int(rng.integers(0, 7)),
        scale_interval_ms=int(rng.choice([7000, 60000])), scale_in_idle_pct=int(rng.choice([0, 10, 50])),
        min_hosts=int(rng.integers(0, h0 + 1)))
    if mode == "closed":
        cfg["flags"] = (cfg["flags"] & ~(tg.F_SCALE_IN | tg.F_AUTOSCALE)) | tg.F_CLOSED_LOOP
    elif mode == "batch":
        grow = cfg["flags"] & tg.F_SCALE_OUT
        cfg.update(flags=tg.F_BATCH_MODE | grow, batch_start_delay_ms=int(rng.choice([0, 40, 15000])))
        if not grow:
            cfg["hosts_max"] = cfg["hosts_initial"]
    elif mode == "auto":
        cfg.update(flags=cfg["flags"] | tg.F_AUTOSCALE, autoscale_f_milli=int(rng.choice([0, 1050, 3000])),
                   scaling_buffer_hosts=int(rng.integers(0, 8)), hosts_max=h0 + 50)
    elif mode == "warm":
        cfg.update(flags=cfg["flags"] | tg.F_WARM_POOL | tg.F_MIGRATE, warm_pool_per_host=int(rng.integers(1, 5)),
                   warm_migration_delay_ms=int(rng.choice([0, 300])), prewarm_delay_ms=int(rng.choice([0, 5000, 60000])))
    g = cfg["gpus_per_host"]
    traces = [(t, d, sk, np.minimum(gp, g).astype(np.uint8)) for t, d, sk, gp in traces]
    caps = [int(rng.choice([300, 1000, 1500, 2000, 4000, 100000])) for _ in range(4)]
    return mode, tg.pack(cfg, traces, [0, 1, 0, 1], caps, f"mid{seed}")


@pytest.mark.parametrize("block", range(6))
def test_mid_size_random_cases(oracle, block):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_20591_amd import replay as rp
    rp.load()
    for seed in range(20 * block, 20 * block + 20):
        mode, b = draw_case(seed)
        dev = rp.upload(b)
        want = []
        for r in range(b.n_replays):
            t = int(b.trace_of_replay[r])
            a, e = int(b.ev_offset[t]), int(b.ev_offset[t + 1])
            sa, sb = int(b.sess_offset[t]), int(b.sess_offset[t + 1])
            want.append(oracle.replay(b.config, b.ev_time[a:e], b.ev_dur[a:e], b.ev_sk[a:e], b.sess_gpus[sa:sb],
                                      int(b.cap_milli[r])))
        for in_lds in ((False, True) if mode != "batch" else (False,)):
            for rounds in ((None, True, False) if in_lds else (None,)):
                h = rp.Replay(b.config, dev, hosts_in_lds=in_lds, rounds=rounds)
                h.run()
                st = h.stats()
                h.close()
                for r in range(b.n_replays):
                    got = rp.stats_to_dict(st[r])
                    assert got["status"] == 0, (seed, mode, in_lds, rounds, r)
                    for k in oracle.RESULT_FIELDS:
                        assert got[k] == want[r][k], (seed, mode, in_lds, rounds, r, k, got[k], want[r][k])
