"""The policy study (paper_2503_20591_amd.sweep) on the GPU: its rows against the oracle, and the
relationships the paper's evaluation reports, on synthetic traces."""
import numpy as np
import pytest

from paper_2503_20591_amd import tracegen as tg

pytestmark = pytest.mark.gpu

CAPS = (1000, 1500, 2000, 3000, 4000)


@pytest.fixture(scope="module")
def study():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_20591_amd import replay, sweep
    replay.load()
    batch = sweep.study_batch(n_traces=2, caps=CAPS, sessions=400, cells=24_000, hosts_initial=8, hosts_max=128)
    return batch, sweep.run_policies(batch, batch_start_delay_ms=15_000)


def test_rows_match_the_oracle(study, oracle):
    batch, rows = study
    assert len(rows) == batch.n_replays == 2 * len(CAPS)
    for r, row in enumerate(rows):
        t = int(batch.trace_of_replay[r])
        a, b = int(batch.ev_offset[t]), int(batch.ev_offset[t + 1])
        sa, sb = int(batch.sess_offset[t]), int(batch.sess_offset[t + 1])
        ev = (batch.ev_time[a:b], batch.ev_dur[a:b], batch.ev_sk[a:b], batch.sess_gpus[sa:sb])
        w = oracle.replay(batch.config, *ev, int(batch.cap_milli[r]))
        assert row["peak_hosts"] == w["peak_hosts"] and row["migrations"] == w["migrations"]
        assert row["provisioned_gpu_h"] == w["gpu_ms_provisioned"] / 3.6e6
        assert row["committed_gpu_h"] == w["gpu_ms_committed"] / 3.6e6
        assert row["reservation_gpu_h"] == w["reservation_gpu_ms"] / 3.6e6
        bill = oracle.billing(w, batch.config["gpus_per_host"], 10_000_000, 115, 125)
        revenue = bill["usage_revenue"] + bill["standby_revenue"]
        assert row["margin"] == (revenue - bill["provider_cost"]) / revenue
        cfg_b = dict(batch.config, flags=tg.F_BATCH_MODE | tg.F_SCALE_OUT, batch_start_delay_ms=15_000)
        wb = oracle.replay(cfg_b, *ev, int(batch.cap_milli[r]))
        assert row["batch_peak_hosts"] == wb["peak_hosts"]
        assert row["batch_mean_delay_s"] == wb["sum_delay_ms"] / max(wb["cells_started"], 1) / 1e3


def test_relationships_of_the_evaluation(study):
    _, rows = study
    for t in range(2):
        by_cap = [x for x in rows if x["trace"] == t]
        assert [x["cap"] for x in by_cap] == [c / 1000 for c in CAPS]
        lo, hi = by_cap[0], by_cap[-1]
        # a higher subscription-ratio cap packs more replicas per host: fewer hosts are provisioned,
        # at the price of more migrations (section "Subscription Ratio")
        assert hi["peak_hosts"] < lo["peak_hosts"] and hi["provisioned_gpu_h"] < lo["provisioned_gpu_h"]
        assert hi["migrations"] > lo["migrations"]
        assert hi["margin"] > lo["margin"]              # and the provider's margin grows (section "Monetary Cost")
        assert all(b["provisioned_gpu_h"] <= 1.02 * a["provisioned_gpu_h"] for a, b in zip(by_cap, by_cap[1:]))
        for x in by_cap:
            # GPUs are bound only while cells run: far fewer GPU-hours than reserving them for the
            # sessions' lifetimes (section "Resource Usage & Efficiency")
            assert x["committed_gpu_h"] < 0.6 * x["reservation_gpu_h"]
            # most cells start at once, and the mean delay stays far below the Batch baseline's, which
            # pays a container start per cell (section "Interactivity")
            assert x["immediate"] > 0.8
            assert x["batch_mean_delay_s"] >= 15.0 and x["mean_delay_s"] < 0.5 * x["batch_mean_delay_s"]
