"""Do the pins bite?  Plant one plausible mistake at a time in a COPY of the oracle's C source
(on the CPU, in a temp dir), rebuild, and require that at least one pin fails."""
import os
import subprocess
import sys
import types

import pytest

import test_oracle_pins as pins
from helpers import GOLDEN

MUTANTS = [
    ("cap: request dropped from the sum", "(h->S + g) * 1000 <=", "(h->S) * 1000 <="),
    ("cap: R dropped from S/(G*R)", "m->p->cap_milli * m->G * R", "m->p->cap_milli * m->G"),
    ("placement prefers MORE committed GPUs", "if (x->C != y->C) return x->C < y->C;",
     "if (x->C != y->C) return x->C > y->C;"),
    ("placement prefers HIGHER subscription", "if (x->S != y->S) return x->S < y->S;",
     "if (x->S != y->S) return x->S > y->S;"),
    ("placement tie to the highest index", "  return a < b;\n}", "  return a > b;\n}"),
    ("election tie to the highest host", "q->host[i] < q->host[lead]", "q->host[i] > q->host[lead]"),
    ("election prefers the fullest host", "if (x->C < y->C || (x->C == y->C && q->host[i] < q->host[lead]))",
     "if (x->C > y->C || (x->C == y->C && q->host[i] < q->host[lead]))"),
    ("election off by one", "if (x->state != H_READY || m->G - x->C < g) continue;\n    if (lead",
     "if (x->state != H_READY || m->G - x->C <= g) continue;\n    if (lead"),
    ("victim is the emptiest host", "if (x->C > y->C || (x->C == y->C && q->host[i] < q->host[victim]))",
     "if (x->C < y->C || (x->C == y->C && q->host[i] < q->host[victim]))"),
    ("timer kinds in reverse order", "if (a->prio != b->prio) return a->prio < b->prio;",
     "if (a->prio != b->prio) return a->prio > b->prio;"),
    ("timers due AT an arrival run after it", "m.heap[0].time <= t && !m.err", "m.heap[0].time < t && !m.err"),
    ("GPUs never released", "release(m, q->host[q->exec_slot], q->g);", ""),
    ("finish ignores the start delay", "int32_t finish = start + q->dur;", "int32_t finish = m->clock + q->dur;"),
    ("migration delay dropped", "start_cell(m, s, victim, m->clock + m->p->migration_delay_ms, ORC_D_MIGRATE)",
     "start_cell(m, s, victim, m->clock, ORC_D_MIGRATE)"),
    ("boot delay dropped for a scaled-out cell", "m->clock + m->p->boot_delay_ms + m->p->migration_delay_ms, ORC_D_SCALE_CELL",
     "m->clock + m->p->migration_delay_ms, ORC_D_SCALE_CELL"),
    ("migration ignores the cap", "if (m->G - x->C < g || !cap_ok(m, x, g)) continue;", "if (m->G - x->C < g) continue;"),
    ("migration forgets to move the subscription", "unsubscribe(m, q->host[victim], g);\n      subscribe(m, dst, g);", "subscribe(m, dst, g);"),
    ("histogram bucket off by one", "for (int32_t x = delay; x > 0; x >>= 1) b++;", "for (int32_t x = delay; x > 1; x >>= 1) b++;"),
    ("scale-in releases 3 per period", "A > m->p->min_hosts && released < 2) {\n    release_empty_host(m);\n    A--; Z--; released++;\n  }\n}",
     "A > m->p->min_hosts && released < 3) {\n    release_empty_host(m);\n    A--; Z--; released++;\n  }\n}"),
    ("scale-in releases the lowest empty host", "int h = m->H - 1;\n  while (!(m->hosts[h].state == H_READY && m->hosts[h].nrep == 0)) h--;",
     "int h = 0;\n  while (!(m->hosts[h].state == H_READY && m->hosts[h].nrep == 0)) h++;"),
    ("auto-scaler: f applied upside down", "(int64_t)m->p->autoscale_f_milli * m->sum_C;", "(int64_t)1000000 / (m->p->autoscale_f_milli + 1) * m->sum_C;"),
    ("auto-scaler: expected capacity rounded down", "(gpus_milli + per_host - 1) / per_host", "gpus_milli / per_host"),
    ("auto-scaler: scaling buffer forgotten", "/ per_host + m->p->scaling_buffer_hosts;", "/ per_host;"),
    ("auto-scaler: uses subscribed instead of committed GPUs", "m->p->autoscale_f_milli * m->sum_C", "m->p->autoscale_f_milli * m->sum_S"),
    ("auto-scaler: per-GPU instead of per-host capacity", "int64_t per_host = (int64_t)1000 * m->G;", "int64_t per_host = (int64_t)1000;"),
    ("auto-scaler: booting hosts not counted as capacity", "while (m->n_on < want && m->n_on < m->H) {", "while (A < want && m->n_on < m->H) { A++;"),
    ("auto-scaler: adds one host per period", "      decide(m, ORC_D_SCALE_AUTO, 0, 0, h);\n    }", "      decide(m, ORC_D_SCALE_AUTO, 0, 0, h);\n      break;\n    }"),
    ("auto-scaler: releases below the expected capacity", "while (m->n_on > want && Z > 0", "while (m->n_on >= want && Z > 0"),
    ("auto-scaler: releases 3 per period", "while (m->n_on > want && Z > 0 && A > m->p->min_hosts && released < 2)",
     "while (m->n_on > want && Z > 0 && A > m->p->min_hosts && released < 3)"),
    ("auto-scaler: ignores min_hosts", "while (m->n_on > want && Z > 0 && A > m->p->min_hosts", "while (m->n_on > want && Z > 0"),
    ("auto-scaler: releases without SCALE_IN", "    if (m->p->flags & ORC_F_SCALE_IN)\n      while (m->n_on > want", "    if (1)\n      while (m->n_on > want"),
    ("auto-scaler never ticks on its own", "if (p->flags & (ORC_F_SCALE_IN | ORC_F_AUTOSCALE)) heap_push", "if (p->flags & ORC_F_SCALE_IN) heap_push"),
    ("dynamic limit: request left out of the cluster sum", "m->n_on <= m->sum_S + g;", "m->n_on <= m->sum_S;"),
    ("dynamic limit: request left out of the host sum", "return (int64_t)(h->S + g) * m->n_on <=", "return (int64_t)(h->S) * m->n_on <="),
    ("dynamic limit: divides by hosts_max", "(h->S + g) * m->n_on <=", "(h->S + g) * m->H <="),
    ("dynamic limit replaces the cap", "if ((int64_t)(h->S + g) * 1000 <= (int64_t)m->p->cap_milli * m->G * R) return 1;\n  /*",
     "if (!(m->p->flags & ORC_F_DYNAMIC_SR) && (int64_t)(h->S + g) * 1000 <= (int64_t)m->p->cap_milli * m->G * R) return 1;\n  /*"),
    ("billing: standby charge not reduced by the executing time", "int64_t standby_ms = r->replica_ms - exec_ms;\n", "int64_t standby_ms = r->replica_ms;\n"),
    ("billing: standby time not clamped at zero", "if (standby_ms < 0) standby_ms = 0;", ""),
    ("billing: markup dropped from the usage charge", "ratio(r->gpu_ms_executed, price * markup_pct, (int64_t)G * ms_per_hour * 100)", "ratio(r->gpu_ms_executed, price * 100, (int64_t)G * ms_per_hour * 100)"),
    ("billing: standby share applied per GPU", "ratio(standby_ms, price * markup_pct * standby_permille, ms_per_hour * 100 * 1000)", "ratio(standby_ms, price * markup_pct * standby_permille, (int64_t)G * ms_per_hour * 100 * 1000)"),
    ("billing: provider cost per GPU-hour", "ratio(r->gpu_ms_provisioned, price, (int64_t)G * ms_per_hour)", "ratio(r->gpu_ms_provisioned, price, ms_per_hour)"),
    ("billing: Reservation billed without markup", "ratio(r->reservation_gpu_ms, price * markup_pct, (int64_t)G * ms_per_hour * 100)", "ratio(r->reservation_gpu_ms, price * 100, (int64_t)G * ms_per_hour * 100)"),
    ("billing: 64-bit product", "(int64_t)((unsigned __int128)amount * (unsigned __int128)num / (unsigned __int128)den)", "(int64_t)((uint64_t)amount * (uint64_t)num / (uint64_t)den)"),
    ("replica integral counts GPUs", "m->r.replica_ms += m->n_replicas * dt;", "m->r.replica_ms += m->sum_S * dt;"),
    ("replicas of ended sessions keep counting", "m->sum_S -= g; m->n_replicas--; }", "m->sum_S -= g; }"),
    ("sticky executor leads although its host is full", "if (x->state == H_READY && m->G - x->C >= g) lead = q->last_exec;", "if (x->state == H_READY) lead = q->last_exec;"),
    ("sticky executor always on", "if ((m->p->flags & ORC_F_STICKY) && lead >= 0 && q->last_exec >= 0) {", "if (lead >= 0 && q->last_exec >= 0) {"),
    ("sticky executor never applied", "if (x->state == H_READY && m->G - x->C >= g) lead = q->last_exec;", ";"),
    ("sticky executor off by one GPU", "if (x->state == H_READY && m->G - x->C >= g) lead = q->last_exec;", "if (x->state == H_READY && m->G - x->C > g) lead = q->last_exec;"),
    ("batch: a later job overtakes the head of the queue", "      return;\n    }\n    /* a long queue", "      m->head = (m->head + 1) % (m->n_sess + 1); m->fifo[(m->head + m->count - 1) % (m->n_sess + 1)] = s;\n      if (++j->asked > m->count + 1) return;\n      continue;\n    }\n    /* a long queue", "nbos_oracle_batch.c"),
    ("batch: container start not part of the delay", "int32_t delay = start - j->t_submit;", "int32_t delay = m->clock - j->t_submit;", "nbos_oracle_batch.c"),
    ("batch: GPUs not held during the container start", "(int64_t)j->g * ((int64_t)finish - m->clock)", "(int64_t)j->g * j->dur", "nbos_oracle_batch.c"),
    ("batch: fullest feasible server", "if (best < 0 || x->C < m->hosts[best].C) best = h;", "if (best < 0 || x->C > m->hosts[best].C) best = h;", "nbos_oracle_batch.c"),
    ("batch: tie to the highest index", "if (best < 0 || x->C < m->hosts[best].C) best = h;", "if (best < 0 || x->C <= m->hosts[best].C) best = h;", "nbos_oracle_batch.c"),
    ("batch: GPUs never given back", "m->hosts[j->host].C -= j->g;", "", "nbos_oracle_batch.c"),
    ("batch: feasibility off by one", "m->G - x->C < j->g) continue;", "m->G - x->C <= j->g) continue;", "nbos_oracle_batch.c"),
    ("batch: busy session's cell is queued anyway", "if (j->state != J_IDLE) { m.r.cells_dropped_busy++; continue; }", "if (j->state == J_QUEUED) { m.r.cells_dropped_busy++; continue; }", "nbos_oracle_batch.c"),
    ("batch: every queued job asks for a server", "j->asked = 1;", "", "nbos_oracle_batch.c"),
    ("batch: timers due at an arrival run after it", "m.heap[0].time <= t && !m.err) run_instant(&m);", "m.heap[0].time < t && !m.err) run_instant(&m);", "nbos_oracle_batch.c"),
    ("batch: queue looked at between two timers of one instant", "    }\n  }\n  dispatch(m);\n}", "    }\n    dispatch(m);\n  }\n  dispatch(m);\n}", "nbos_oracle_batch.c"),
    ("warm pool: takes the newest container", "if (d->warm[i] < d->warm[w]) w = i;", "if (d->warm[i] > d->warm[w]) w = i;"),
    ("warm pool: never refilled", "d->warm[w] = m->clock + m->p->prewarm_delay_ms;", "d->warm[w] = 2147483647;"),
    ("warm pool: refilled at once", "d->warm[w] = m->clock + m->p->prewarm_delay_ms;", ""),
    ("warm pool: an added host is warm from the start", "m->hosts[h].warm[i] = m->hosts[h].ready_at + m->p->prewarm_delay_ms;", "m->hosts[h].warm[i] = 0;"),
    ("warm pool: container available exactly now is not taken", "if (d->warm[w] <= m->clock) {", "if (d->warm[w] < m->clock) {"),
    ("warm pool: warm start pays the cold delay", "m->clock + m->p->warm_migration_delay_ms, ORC_D_MIGRATE_WARM", "m->clock + m->p->migration_delay_ms, ORC_D_MIGRATE_WARM"),
    ("warm pool: only one container per host", "for (int i = 1; i < m->p->warm_pool_per_host; i++)", "for (int i = 1; i < 1; i++)"),
    ("closed loop: think measured from the previous event's start", "anchor[s] = kind == ORC_EV_CELL ? ev_time[i] + ev_dur[i] : ev_time[i];", "anchor[s] = ev_time[i];"),
    ("closed loop: next event counted from the start of the cell", "if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, finish);", "if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, start);"),
    ("closed loop: a cell that is given up ends the chain", "  if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, m->clock);\n}\n\nstatic void on_cell", "}\n\nstatic void on_cell"),
    ("closed loop: first cell counted from time 0", "  m->r.sessions_placed++;\n  if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, m->clock);", "  m->r.sessions_placed++;\n  if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, 0);"),
    ("closed loop: think time of the END ignored", "      m.think[i] = ev_time[i] > anchor[s] ? ev_time[i] - anchor[s] : 0;", "      m.think[i] = (kind == ORC_EV_END) ? 0 : (ev_time[i] > anchor[s] ? ev_time[i] - anchor[s] : 0);"),
    ("closed loop: due events run before retries of the same instant", "enum { T_COMPLETE = 0, T_HOST_READY = 1, T_RETRY = 2, T_NEXT = 3, T_TICK = 4 };", "enum { T_COMPLETE = 0, T_HOST_READY = 1, T_RETRY = 3, T_NEXT = 2, T_TICK = 4 };"),
    ("closed loop: cells keep their time in the trace", "    if (closed && !first_start[i]) continue;", "    if (0) continue;"),
    ("dynamic limit always on", "if (m->p->flags & ORC_F_DYNAMIC_SR)\n    return", "if (1)\n    return"),
    ("Reservation ignores END", "q->has_end ? q->end_time : m.clock", "m.clock"),
    ("executor reuse inverted", "if (q->last_exec == slot)", "if (q->last_exec != slot)"),
    ("scale-out not all-or-nothing", "m->n_on + missing <= m->H", "m->n_on < m->H"),
    ("every start counted immediate", "if (m->clock == q->t_submit) m->r.cells_immediate++;", "m->r.cells_immediate++;"),
    ("END while busy ends at once", "if (!q->ending) { q->ending = 1; q->has_end = 1; q->end_time = m->clock; }",
     "q->has_end = 1; q->end_time = m->clock; end_session(m, s);"),
    ("retry budget off by one", "if (q->retries < m->p->max_retries) {", "if (q->retries <= m->p->max_retries) {"),
    ("tick keeps running after the last timer", "if (m.heap[0].prio == T_TICK && m.n_heap == 1) break;",
     "if (m.heap[0].prio == T_TICK && m.n_heap == 1 && m.clock > 100000000) break;"),
    ("booting host takes part in elections", "if (x->state != H_READY || m->G - x->C < g) continue;\n    if (lead",
     "if (x->state == H_OFF || m->G - x->C < g) continue;\n    if (lead"),
    ("subscribed integral uses committed GPUs", "m->r.sub_gpu_ms += m->sum_S * dt;", "m->r.sub_gpu_ms += m->sum_C * dt;"),
    ("provisioned integral ignores G", "(int64_t)m->n_on * m->G * dt", "(int64_t)m->n_on * dt"),
    ("tct measured from the start", "m->r.sum_tct_ms += (int64_t)finish - q->t_submit;", "m->r.sum_tct_ms += (int64_t)finish - start;"),
]


def _shim(orc, lib_path):
    ns = types.SimpleNamespace(**{k: getattr(orc, k) for k in dir(orc) if k.startswith(("D_", "F_", "EV_"))})
    ns.decode = orc.decode
    ns.RESULT_FIELDS = orc.RESULT_FIELDS
    ns.billing = lambda *a, **kw: orc.billing(*a, lib_path=lib_path, **kw)
    ns.replay = lambda *a, **kw: orc.replay(*a, lib_path=lib_path, **kw)

    def replay_batch(batch, replays=None, check=False, threads=1):
        out = []
        for r in (range(batch.n_replays) if replays is None else replays):
            t = int(batch.trace_of_replay[r])
            a, b = int(batch.ev_offset[t]), int(batch.ev_offset[t + 1])
            sa, sb = int(batch.sess_offset[t]), int(batch.sess_offset[t + 1])
            out.append(ns.replay(batch.config, batch.ev_time[a:b], batch.ev_dur[a:b], batch.ev_sk[a:b],
                                 batch.sess_gpus[sa:sb], int(batch.cap_milli[r]), check=check))
        return out
    ns.replay_batch = replay_batch
    return ns


def run_pins(lib_path):
    """Exit status 0 iff every pin accepts the oracle build at lib_path (runs in a child process)."""
    import oracle as orc
    o = _shim(orc, lib_path)
    checks = [lambda: pins.test_sr_worked_example(o), lambda: pins.test_sr_counts_idle_replicas_and_uses_R(o)]
    checks += [lambda n=n: pins.test_hand_worked(o, n) for n in sorted(os.listdir(GOLDEN)) if n.startswith("hand_")]
    checks += [lambda: pins.test_placement_brute_force(o), lambda: pins.test_election_brute_force(o),
               lambda: pins.test_no_contention_closed_form(o), lambda: pins.test_single_session_textbook(o),
               lambda: pins.test_reservation_and_subscription_closed_form(o)]
    checks += [lambda s=s: pins.test_invariants_random(o, s) for s in range(12)]
    for args in [(1050, 0, 1), (1050, 2, 1), (1050, 0, 3), (3000, 0, 2), (4100, 5, 3), (0, 4, 3)]:
        checks.append(lambda a=args: pins.test_autoscale_adds_up_to_expected_capacity(o, *a))
    for args in [(0, 0, [(1000, 8), (1000, 7), (2000, 6), (2000, 5), (3000, 4), (3000, 3)]),
                 (0, 6, [(1000, 8), (1000, 7), (2000, 6)]), (5, 0, [(1000, 8), (1000, 7), (2000, 6)])]:
        checks.append(lambda a=args: pins.test_autoscale_releases_two_per_tick_down_to_capacity(o, *a))
    checks += [lambda s=s: pins.test_autoscale_with_f_zero_is_the_plain_policy(o, s) for s in range(6)]
    checks += [lambda s=s: pins.test_dynamic_limit_is_vacuous_on_large_clusters(o, s) for s in range(8)]
    checks.append(lambda: pins.test_dynamic_limit_brute_force(o))
    checks.append(lambda: pins.test_sticky_election_brute_force(o))
    checks += [lambda: pins.test_warm_pool_pin_sees_many_migrations(o)]
    checks += [lambda s=s: pins.test_closed_loop_without_waiting_is_the_open_loop(o, s) for s in range(3)]
    checks += [lambda s=s: pins.test_closed_loop_schedule_from_the_log(o, s) for s in range(5)]
    checks += [lambda s=s: pins.test_closed_loop_never_meets_a_busy_session(o, s) for s in range(4)]
    checks += [lambda s=s: pins.test_warm_pool_that_refills_at_once_is_a_shorter_delay(o, s) for s in range(3)]
    checks += [lambda: pins.test_batch_single_server_is_the_textbook_fifo_queue(o), lambda: pins.test_batch_without_contention(o)]
    checks += [lambda s=s: pins.test_batch_order_and_capacity_random(o, s) for s in range(6)]
    checks += [lambda: pins.test_billing_printed_example(o), lambda: pins.test_billing_is_linear_and_exact_on_large_results(o),
               lambda: pins.test_billing_without_replicas_has_no_standby_charge(o)]
    checks += [lambda s=s: pins.test_replica_integral_random(o, s) for s in range(3)]
    for c in checks:
        try:
            c()
        except (AssertionError, ValueError, KeyError, IndexError):
            return 1
    return 0


def _pins_fail(lib_path):
    here = os.path.dirname(os.path.abspath(__file__))
    code = ("import sys; sys.path[:0] = [%r, %r]; import test_oracle_mutants as t; sys.exit(t.run_pins(%r))"
            % (here, os.path.dirname(here), lib_path))
    try:
        rc = subprocess.run([sys.executable, "-c", code], timeout=120, stdout=subprocess.DEVNULL,
                            stderr=subprocess.DEVNULL).returncode
    except subprocess.TimeoutExpired:
        return True
    return rc != 0


SOURCES = ("nbos_oracle.c", "nbos_oracle_batch.c")


def _build(oracle, tmp_path, name, edit):
    """Copy the oracle's sources to tmp_path, passing the text of each through edit(file, text)."""
    odir = os.path.dirname(oracle.__file__)
    for f in SOURCES:
        (tmp_path / f).write_text(edit(f, open(os.path.join(odir, f)).read()))
    (tmp_path / "nbos_oracle.h").write_text(open(os.path.join(odir, "nbos_oracle.h")).read())
    out = str(tmp_path / name)
    subprocess.run(["gcc", "-std=c99", "-O1", "-w", "-fPIC", "-shared", "-o", out, *SOURCES],
                   check=True, cwd=tmp_path)
    return out


def test_unmutated_copy_passes(oracle, tmp_path):
    assert not _pins_fail(_build(oracle, tmp_path, "clean.so", lambda f, s: s))


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(oracle, tmp_path, idx):
    name, old, new = MUTANTS[idx][:3]
    target = MUTANTS[idx][3] if len(MUTANTS[idx]) > 3 else SOURCES[0]

    def edit(f, src):
        if f != target:
            return src
        assert src.count(old) >= 1, f"mutation site gone: {name}"
        return src.replace(old, new, 1)
    assert _pins_fail(_build(oracle, tmp_path, f"mutant{idx}.so", edit)), f"no pin notices: {name}"
