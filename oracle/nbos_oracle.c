/*
 * nbos_oracle.c — CPU oracle of the NotebookOS policy replay.
 *
 * TEST INFRASTRUCTURE. Plain C99, single-threaded, eager discrete-event loop:
 * one pending-timer set, every timer processed at its own time, every state
 * change applied when it happens. No blocking, batching or lazy evaluation.
 * Only tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What each part follows (paper section):
 *   host record G / C / S and the subscription ratio S/(G*R) ....... 3.4.1
 *   placement of R = 3 replicas on distinct least-loaded hosts ..... 3.2.1, 3.4.1
 *   executor election by outcome (LEAD if the host can bind GPUs) .. 3.2.2
 *   dynamic GPU binding: commit at start, release at completion .... 3.3
 *   failed election -> migration, retry queue, abort ............... 3.2.3
 *   scale-out on failed placement, periodic scale-in ............... 3.4.2
 *   auto-scaler: expected capacity f * sum C, scaling buffer ....... 3.4.2
 *   dynamic cluster-wide limit on the subscription ratio ........... 3.4.1
 *   metric definitions (delay, TCT, immediate, reuse, GPU-hours) ... "Resource Usage & Efficiency", "Interactivity", "Task Completion Time"
 *   billing model (provider cost, revenue, standby charge) ......... "Monetary Cost"
 *   pre-warmed container pool for migrations ........................ 3.2.3
 *
 * Readings taken where the paper leaves a choice open (all deterministic):
 *   - host preference key, smaller is better: (committed GPUs, subscribed GPUs,
 *     host index). "More idle GPUs first" with uniform G is "fewer committed".
 *   - cap test for a replica with request g on host h:
 *         (S_h + g) * 1000 <= cap_milli * G * 3
 *   - the elected executor is the feasible replica on the host with the fewest
 *     committed GPUs, ties to the lowest host index.
 *   - the migrated replica is the one on the host with the most committed GPUs
 *     (ties: lowest host index); replicas on booting hosts only if all three are.
 *   - a scaled-out host is reserved for the replicas that caused it until ready.
 *   - a cell arriving while its session is busy is dropped and counted.
 *   - timers due at the same time run in the order COMPLETE, HOST_READY, RETRY,
 *     TICK, then by ascending session / host id; all timers due at or before an
 *     arrival run before it; arrivals keep input order.
 *   - a TICK runs only while an arrival or another timer is still pending.
 *   - auto-scaler (ORC_F_AUTOSCALE): at every TICK the expected capacity is
 *     want = ceil(f * sum C / G) + buffer hosts, sum C = GPUs committed at that
 *     instant. Hosts that are booting count as capacity. Below want: boot the
 *     difference at once (lowest unused indices, up to hosts_max). With
 *     ORC_F_SCALE_IN also set and more than want hosts provisioned: release at
 *     most 2 ready hosts without replicas per TICK, highest index first, never
 *     below want or min_hosts (so a release is never undone by the next TICK).
 *   - dynamic limit (ORC_F_DYNAMIC_SR): a host also passes the cap test when its
 *     ratio after taking the replica is at most the cluster-wide ratio after
 *     taking it, (S_h + g) / (G R) <= (sum S + g) / (n G R), n = hosts not off;
 *     i.e. the limit in force is the larger of the configured cap and that mean.
 *   - pre-warmed containers (ORC_F_WARM_POOL): every host keeps warm_pool_per_host of
 *     them; an initial host has them from time 0, a provisioned host prewarm_delay_ms
 *     after it is ready. A migration takes the target's container that has been
 *     available longest, if one is available now: the cell then starts after
 *     warm_migration_delay_ms instead of migration_delay_ms, and a replacement is
 *     available prewarm_delay_ms later. A host added for the cell has none yet.
 *   - closed loop (ORC_F_CLOSED_LOOP; the section "Interactive Deep Learning Training" describes users who think, edit and
 *     re-submit between cells): only a session's first START keeps its time. Every
 *     later CELL / END of the session is due one think time after the session's
 *     previous cell is over (finished or given up; for the first one: after the
 *     placement), where the think time is what the trace leaves between the
 *     previous event's nominal end (its time, plus its duration for a CELL) and the
 *     event's own time, at least 0. Events before the first START, repeated STARTs
 *     and everything after the first END are ignored. Due events run as timers
 *     after RETRY timers of the same instant, by ascending session id. No cell
 *     ever meets a busy session. Not combined with the periodic auto-scaler.
 *   - sticky executor (ORC_F_STICKY): when the replica that executed the session's
 *     previous cell can lead (host ready, enough idle GPUs) it does; else the rule above.
 */
#include "nbos_oracle.h"
#include <stdlib.h>
#include <string.h>

#define R 3
#define MAX_DUR 86400000

enum { H_OFF = 0, H_BOOT = 1, H_READY = 2 };
enum { S_UNPLACED = 0, S_IDLE = 1, S_BUSY = 2, S_REJECTED = 3, S_ENDED = 4 };
enum { T_COMPLETE = 0, T_HOST_READY = 1, T_RETRY = 2, T_NEXT = 3, T_TICK = 4 };

typedef struct { int32_t time; int32_t prio; int32_t id; } tmr;

typedef struct {
  int state;
  int32_t ready_at;
  int C, S, nrep;
  int32_t warm[4];    /* when each pre-warmed container is (again) available */
} host_rec;

typedef struct {
  int state;
  int host[R];
  int g;
  int last_exec;      /* -1 none, else replica slot of the previous executed cell */
  int ending;         /* END seen while busy: end when the cell is over           */
  int has_end;        /* an END event was accepted                                */
  int32_t end_time;   /* its time                                                 */
  int32_t t_placed;   /* time of the accepted START                               */
  int32_t t_submit, dur;
  int retries;
  int exec_slot;      /* -1 while queued                                          */
  int queued_once;
} sess_rec;

typedef struct {
  const orc_params *p;
  int H, G;
  host_rec *hosts;
  sess_rec *sess;
  int n_sess;
  tmr *heap; int n_heap, cap_heap;
  int32_t clock;
  int n_on;                 /* hosts not off        */
  int64_t sum_S, sum_C;     /* cluster totals       */
  int64_t n_replicas;       /* placed replicas      */
  orc_result r;
  uint64_t *log; int64_t log_cap;
  /* self-check accumulators */
  int64_t chk_commit_integral, chk_wait_gpu_ms;
  uint32_t chk_starts_seen;
  tmr last_popped; int have_last;
  int err;
  /* closed loop: the trace, each session's chain of events and where it stands */
  const int32_t *ev_dur, *ev_sk;
  int32_t *think;           /* [n_events] think time before the event       */
  int64_t *next_ev;         /* [n_events] next event of the same session, -1 */
  int64_t *cursor;          /* [n_sess] the session's next event, -1 = none  */
} sim;

/* ---- pending timers: textbook binary min-heap on (time, prio, id) ---------- */
static int tmr_less(const tmr *a, const tmr *b) {
  if (a->time != b->time) return a->time < b->time;
  if (a->prio != b->prio) return a->prio < b->prio;
  return a->id < b->id;
}
static void heap_push(sim *m, int32_t time, int prio, int id) {
  if (m->n_heap == m->cap_heap) {
    int nc = m->cap_heap * 2;
    tmr *nh = (tmr *)realloc(m->heap, (size_t)nc * sizeof(tmr));
    if (!nh) { m->err = ORC_E_NOMEM; return; }
    m->heap = nh; m->cap_heap = nc;
  }
  int i = m->n_heap++;
  tmr t = { time, prio, id };
  while (i > 0) {
    int par = (i - 1) / 2;
    if (!tmr_less(&t, &m->heap[par])) break;
    m->heap[i] = m->heap[par];
    i = par;
  }
  m->heap[i] = t;
}
static tmr heap_pop(sim *m) {
  tmr top = m->heap[0];
  tmr last = m->heap[--m->n_heap];
  int i = 0;
  for (;;) {
    int c = 2 * i + 1;
    if (c >= m->n_heap) break;
    if (c + 1 < m->n_heap && tmr_less(&m->heap[c + 1], &m->heap[c])) c++;
    if (!tmr_less(&m->heap[c], &last)) break;
    m->heap[i] = m->heap[c];
    i = c;
  }
  if (m->n_heap > 0) m->heap[i] = last;
  return top;
}

/* ---- bookkeeping ----------------------------------------------------------- */
static void decide(sim *m, int outcome, int s, int slot, int host) {
  uint64_t code = (uint64_t)(uint32_t)host | ((uint64_t)slot << 10) |
                  ((uint64_t)outcome << 12) | ((uint64_t)s << 16) |
                  ((uint64_t)(uint32_t)m->clock << 32);
  m->r.digest = m->r.digest * 0x100000001B3ULL + code;
  if (m->log && (int64_t)m->r.n_decisions < m->log_cap) m->log[m->r.n_decisions] = code;
  m->r.n_decisions++;
}

/* Move the clock; the integrals of provisioned and subscribed GPUs grow with it. */
static void advance(sim *m, int32_t t) {
  int64_t dt = (int64_t)t - m->clock;
  m->r.gpu_ms_provisioned += (int64_t)m->n_on * m->G * dt;
  m->r.sub_gpu_ms += m->sum_S * dt;
  m->r.replica_ms += m->n_replicas * dt;
  m->chk_commit_integral += m->sum_C * dt;
  m->clock = t;
}

static int cap_ok(const sim *m, const host_rec *h, int g) {
  if ((int64_t)(h->S + g) * 1000 <= (int64_t)m->p->cap_milli * m->G * R) return 1;
  /* Section 3.4.1, third factor: the cluster-wide ratio sum S / (sum G * R) as the limit */
  if (m->p->flags & ORC_F_DYNAMIC_SR)
    return (int64_t)(h->S + g) * m->n_on <= m->sum_S + g;
  return 0;
}

/* preference among hosts: fewer committed, then fewer subscribed, then lower index */
static int host_better(const sim *m, int a, int b) {
  const host_rec *x = &m->hosts[a], *y = &m->hosts[b];
  if (x->C != y->C) return x->C < y->C;
  if (x->S != y->S) return x->S < y->S;
  return a < b;
}

static void subscribe(sim *m, int h, int g) { m->hosts[h].S += g; m->hosts[h].nrep++; m->sum_S += g; m->n_replicas++; }
static void unsubscribe(sim *m, int h, int g) { m->hosts[h].S -= g; m->hosts[h].nrep--; m->sum_S -= g; m->n_replicas--; }
static void commit(sim *m, int h, int g) { m->hosts[h].C += g; m->sum_C += g; }
static void release(sim *m, int h, int g) { m->hosts[h].C -= g; m->sum_C -= g; }

/* Section 3.4.2: provision the lowest-numbered unused host; ready after the boot delay. */
static int boot_host(sim *m) {
  for (int h = 0; h < m->H; h++) {
    if (m->hosts[h].state == H_OFF) {
      m->hosts[h].state = H_BOOT;
      m->hosts[h].ready_at = m->clock + m->p->boot_delay_ms;
      for (int i = 0; i < 4; i++)          /* its pool is filled once it is up */
        m->hosts[h].warm[i] = m->hosts[h].ready_at + m->p->prewarm_delay_ms;
      m->n_on++;
      if ((uint32_t)m->n_on > m->r.peak_hosts) m->r.peak_hosts = (uint32_t)m->n_on;
      heap_push(m, m->hosts[h].ready_at, T_HOST_READY, h);
      return h;
    }
  }
  return -1;
}

/* closed loop: the session's next event is due one think time after `base` */
static void schedule_next(sim *m, int s, int32_t base) {
  int64_t e = m->cursor[s];
  if (e < 0) return;
  int64_t t = (int64_t)base + m->think[e];
  if (t >= 2147483647LL) { m->err = ORC_E_INPUT; return; }     /* beyond the int32 time range */
  heap_push(m, (int32_t)t, T_NEXT, s);
}

/* ---- SESSION_START: Sections 3.2.1, 3.4.1, 3.4.2 ---------------------------- */
static void on_session_start(sim *m, int s) {
  sess_rec *q = &m->sess[s];
  if (q->state != S_UNPLACED) return;
  int g = q->g, pick[R], k = 0;
  for (int i = 0; i < R; i++) {
    int best = -1;
    for (int h = 0; h < m->H; h++) {
      const host_rec *x = &m->hosts[h];
      if (x->state != H_READY || m->G < g || !cap_ok(m, x, g)) continue;
      int taken = 0;
      for (int j = 0; j < k; j++) if (pick[j] == h) taken = 1;
      if (taken) continue;
      if (best < 0 || host_better(m, h, best)) best = h;
    }
    if (best < 0) break;
    pick[k++] = best;
  }
  int missing = R - k;
  if (missing > 0 && !((m->p->flags & ORC_F_SCALE_OUT) && m->n_on + missing <= m->H)) {
    q->state = S_REJECTED;
    m->r.sessions_rejected++;
    decide(m, ORC_D_REJECT, s, 0, 0);
    return;
  }
  for (int i = 0; i < k; i++) {
    q->host[i] = pick[i];
    subscribe(m, pick[i], g);
    decide(m, ORC_D_PLACE, s, i, pick[i]);
  }
  for (int i = k; i < R; i++) {           /* resources reserved before the host is up */
    int h = boot_host(m);
    q->host[i] = h;
    subscribe(m, h, g);
    m->r.scale_out_hosts++;
    decide(m, ORC_D_PLACE_NEW, s, i, h);
  }
  q->state = S_IDLE;
  q->t_placed = m->clock;
  m->r.sessions_placed++;
  if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, m->clock);
}

/* ---- a cell starts: Section 3.3 (bind GPUs), metrics of sections "Resource Usage & Efficiency", "Interactivity" and "Task Completion Time" - */
static void start_cell(sim *m, int s, int slot, int32_t start, int outcome) {
  sess_rec *q = &m->sess[s];
  int32_t commit_t = m->clock;
  if ((int64_t)start + q->dur >= 2147483647LL) { m->err = ORC_E_INPUT; return; }   /* closed loop only */
  int32_t finish = start + q->dur;
  int32_t delay = start - q->t_submit;
  q->exec_slot = slot;
  heap_push(m, finish, T_COMPLETE, s);
  m->r.cells_started++;
  m->r.sum_delay_ms += delay;
  if (delay > m->r.max_delay_ms) m->r.max_delay_ms = delay;
  int b = 0;
  for (int32_t x = delay; x > 0; x >>= 1) b++;       /* 0 -> 0, else 1 + floor(log2) */
  if (b > 31) b = 31;
  m->r.delay_hist[b]++;
  m->r.sum_tct_ms += (int64_t)finish - q->t_submit;
  m->r.gpu_ms_executed += (int64_t)q->g * q->dur;
  m->r.gpu_ms_committed += (int64_t)q->g * ((int64_t)finish - commit_t);
  m->chk_wait_gpu_ms += (int64_t)q->g * ((int64_t)start - commit_t);
  if (q->last_exec == slot) m->r.executor_reused++;
  q->last_exec = slot;
  decide(m, outcome, s, slot, q->host[slot]);
  if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, finish);
}

static void end_session(sim *m, int s) {
  sess_rec *q = &m->sess[s];
  for (int i = 0; i < R; i++) unsubscribe(m, q->host[i], q->g);
  q->state = S_ENDED;
}

/* ---- one attempt to run the pending cell of session s at the current time ----- */
static void attempt(sim *m, int s) {
  sess_rec *q = &m->sess[s];
  int g = q->g;
  /* (a) election, Section 3.2.2: a replica leads iff its host can bind g GPUs now */
  int lead = -1;
  for (int i = 0; i < R; i++) {
    const host_rec *x = &m->hosts[q->host[i]];
    if (x->state != H_READY || m->G - x->C < g) continue;
    if (lead < 0) { lead = i; continue; }
    const host_rec *y = &m->hosts[q->host[lead]];
    if (x->C < y->C || (x->C == y->C && q->host[i] < q->host[lead])) lead = i;
  }
  /* variant: the replica that ran the previous cell keeps leading while its host can bind */
  if ((m->p->flags & ORC_F_STICKY) && lead >= 0 && q->last_exec >= 0) {
    const host_rec *x = &m->hosts[q->host[q->last_exec]];
    if (x->state == H_READY && m->G - x->C >= g) lead = q->last_exec;
  }
  if (lead >= 0) {
    commit(m, q->host[lead], g);
    if (m->clock == q->t_submit) m->r.cells_immediate++;
    start_cell(m, s, lead, m->clock, ORC_D_START);
    return;
  }
  /* every replica yields: choose the replica that would move */
  int any_ready = 0;
  for (int i = 0; i < R; i++) if (m->hosts[q->host[i]].state == H_READY) any_ready = 1;
  int victim = -1;
  for (int i = 0; i < R; i++) {
    const host_rec *x = &m->hosts[q->host[i]];
    if (any_ready && x->state != H_READY) continue;
    if (victim < 0) { victim = i; continue; }
    const host_rec *y = &m->hosts[q->host[victim]];
    if (x->C > y->C || (x->C == y->C && q->host[i] < q->host[victim])) victim = i;
  }
  /* (b) migration, Section 3.2.3: target must bind the GPUs immediately */
  if (m->p->flags & ORC_F_MIGRATE) {
    int dst = -1;
    for (int h = 0; h < m->H; h++) {
      const host_rec *x = &m->hosts[h];
      if (x->state != H_READY) continue;
      if (h == q->host[0] || h == q->host[1] || h == q->host[2]) continue;
      if (m->G - x->C < g || !cap_ok(m, x, g)) continue;
      if (dst < 0 || host_better(m, h, dst)) dst = h;
    }
    if (dst >= 0) {
      unsubscribe(m, q->host[victim], g);
      subscribe(m, dst, g);
      commit(m, dst, g);
      q->host[victim] = dst;
      m->r.migrations++;
      /* Section 3.2.3, pre-warmed container pool: a warm container on the target cuts the delay */
      if (m->p->flags & ORC_F_WARM_POOL) {
        host_rec *d = &m->hosts[dst];
        int w = 0;
        for (int i = 1; i < m->p->warm_pool_per_host; i++) if (d->warm[i] < d->warm[w]) w = i;
        if (d->warm[w] <= m->clock) {
          d->warm[w] = m->clock + m->p->prewarm_delay_ms;
          m->r.migrations_warm++;
          start_cell(m, s, victim, m->clock + m->p->warm_migration_delay_ms, ORC_D_MIGRATE_WARM);
          return;
        }
      }
      start_cell(m, s, victim, m->clock + m->p->migration_delay_ms, ORC_D_MIGRATE);
      return;
    }
  }
  /* (c) scale-out for the cell, Section 3.4.2: reserve on the new host at once */
  if ((m->p->flags & ORC_F_SCALE_OUT) && m->n_on < m->H) {
    unsubscribe(m, q->host[victim], g);
    int h = boot_host(m);
    subscribe(m, h, g);
    commit(m, h, g);
    q->host[victim] = h;
    m->r.scale_out_hosts++;
    m->r.migrations++;
    start_cell(m, s, victim,
               m->clock + m->p->boot_delay_ms + m->p->migration_delay_ms, ORC_D_SCALE_CELL);
    return;
  }
  /* (d) queue and retry periodically, then abort, Section 3.2.3 */
  if (q->retries < m->p->max_retries) {
    q->retries++;
    if (!q->queued_once) { q->queued_once = 1; m->r.cells_queued++; }
    if ((int64_t)q->t_submit + (int64_t)q->retries * m->p->retry_interval_ms >= 2147483647LL) { m->err = ORC_E_INPUT; return; }
    heap_push(m, q->t_submit + q->retries * m->p->retry_interval_ms, T_RETRY, s);
    return;
  }
  q->state = S_IDLE;
  m->r.cells_aborted++;
  decide(m, ORC_D_ABORT, s, 0, 0);
  if (q->ending) end_session(m, s);
  if (m->p->flags & ORC_F_CLOSED_LOOP) schedule_next(m, s, m->clock);
}

static void on_cell(sim *m, int s, int32_t dur) {
  sess_rec *q = &m->sess[s];
  m->r.cells_total++;
  if (q->state == S_BUSY) { m->r.cells_dropped_busy++; return; }
  if (q->state != S_IDLE) { m->r.cells_dropped_unplaced++; return; }
  q->state = S_BUSY;
  q->t_submit = m->clock;
  q->dur = dur;
  q->retries = 0;
  q->queued_once = 0;
  q->exec_slot = -1;
  attempt(m, s);
}

static void on_session_end(sim *m, int s) {
  sess_rec *q = &m->sess[s];
  if (q->state == S_BUSY) {
    if (!q->ending) { q->ending = 1; q->has_end = 1; q->end_time = m->clock; }
  } else if (q->state == S_IDLE) {
    q->has_end = 1; q->end_time = m->clock;
    end_session(m, s);
  }
}

/* ---- timers ---------------------------------------------------------------- */
static void on_complete(sim *m, int s) {
  sess_rec *q = &m->sess[s];
  release(m, q->host[q->exec_slot], q->g);       /* Section 3.3: GPUs released */
  q->state = S_IDLE;
  q->exec_slot = -1;
  if (q->ending) end_session(m, s);
}

/* Release the highest-numbered ready host that holds no replica. */
static void release_empty_host(sim *m) {
  int h = m->H - 1;
  while (!(m->hosts[h].state == H_READY && m->hosts[h].nrep == 0)) h--;
  m->hosts[h].state = H_OFF;
  m->n_on--;
  m->r.scale_in_hosts++;
  decide(m, ORC_D_SCALE_IN, 0, 0, h);
}

/* Section 3.4.2: the periodic auto-scaler. */
static void on_tick(sim *m) {
  int A = 0, Z = 0, released = 0;
  for (int h = 0; h < m->H; h++)
    if (m->hosts[h].state == H_READY) { A++; if (m->hosts[h].nrep == 0) Z++; }
  if (m->p->flags & ORC_F_AUTOSCALE) {
    /* expected capacity sum G' = f * sum C, in whole hosts, plus the scaling buffer */
    int64_t gpus_milli = (int64_t)m->p->autoscale_f_milli * m->sum_C;
    int64_t per_host = (int64_t)1000 * m->G;
    int64_t want = (gpus_milli + per_host - 1) / per_host + m->p->scaling_buffer_hosts;
    while (m->n_on < want && m->n_on < m->H) {
      int h = boot_host(m);
      m->r.scale_out_hosts++;
      decide(m, ORC_D_SCALE_AUTO, 0, 0, h);
    }
    if (m->p->flags & ORC_F_SCALE_IN)
      while (m->n_on > want && Z > 0 && A > m->p->min_hosts && released < 2) {
        release_empty_host(m);
        A--; Z--; released++;
      }
    return;
  }
  /* without the capacity test: release while too large a share of the hosts is empty */
  while ((int64_t)Z * 100 > (int64_t)A * m->p->scale_in_idle_pct &&
         A > m->p->min_hosts && released < 2) {
    release_empty_host(m);
    A--; Z--; released++;
  }
}

/* ---- self-checks (check != 0): structural invariants after every item ------- */
static void verify(sim *m) {
  int H = m->H;
  int *C = (int *)calloc((size_t)H * 3, sizeof(int));
  if (!C) { m->err = ORC_E_NOMEM; return; }
  int *S = C + H, *N = C + 2 * H;
  int bad = 0;
  for (int s = 0; s < m->n_sess && !bad; s++) {
    const sess_rec *q = &m->sess[s];
    if (q->state != S_IDLE && q->state != S_BUSY) continue;
    if (q->host[0] == q->host[1] || q->host[0] == q->host[2] || q->host[1] == q->host[2]) bad = 4;
    for (int i = 0; i < R; i++) {
      int h = q->host[i];
      if (h < 0 || h >= H || m->hosts[h].state == H_OFF) { bad = 4; break; }
      S[h] += q->g; N[h]++;
    }
    if (q->state == S_BUSY && q->exec_slot >= 0) C[q->host[q->exec_slot]] += q->g;
  }
  int n_on = 0; int64_t sS = 0, sC = 0;
  for (int h = 0; h < H && !bad; h++) {
    const host_rec *x = &m->hosts[h];
    if (x->C < 0 || x->C > m->G) bad = 1;
    else if (x->C != C[h]) bad = 2;
    else if (x->S != S[h] || x->nrep != N[h]) bad = 3;
    else if (x->state == H_OFF && (x->S || x->C || x->nrep)) bad = 5;
    if (x->state != H_OFF) n_on++;
    sS += x->S; sC += x->C;
  }
  if (!bad && (n_on != m->n_on || sS != m->sum_S || sC != m->sum_C)) bad = 6;
  free(C);
  if (bad) m->err = ORC_E_INVARIANT - bad;
}

static void run_timer(sim *m, tmr t) {
  if (m->p->check) {
    /* the heap must hand timers out in non-decreasing (time, prio, id) order per
       clock position, and agree with a linear scan for the minimum */
    if (t.time < m->clock) m->err = ORC_E_INVARIANT - 7;
    for (int i = 0; i < m->n_heap; i++)
      if (tmr_less(&m->heap[i], &t)) m->err = ORC_E_INVARIANT - 7;
  }
  advance(m, t.time);
  switch (t.prio) {
    case T_COMPLETE:   on_complete(m, t.id); break;
    case T_HOST_READY: m->hosts[t.id].state = H_READY; break;
    case T_RETRY:      attempt(m, t.id); break;
    case T_NEXT: {                                   /* closed loop: the session's next event is due */
      int64_t e = m->cursor[t.id];
      m->cursor[t.id] = m->next_ev[e];
      if ((int)((uint32_t)m->ev_sk[e] >> 24) == ORC_EV_CELL) on_cell(m, t.id, m->ev_dur[e]);
      else { on_session_end(m, t.id); m->cursor[t.id] = -1; }
      break;
    }
    case T_TICK:
      on_tick(m);
      heap_push(m, t.time + m->p->scale_interval_ms, T_TICK, 0);
      break;
  }
  if (m->p->check && !m->err) verify(m);
}

static int validate(const orc_params *p, int64_t n_events, const int32_t *ev_time,
                    const int32_t *ev_dur, const int32_t *ev_sk, int32_t n_sessions,
                    const uint8_t *sess_gpus) {
  if (p->hosts_initial < 1 || p->hosts_max < p->hosts_initial || p->hosts_max > 1024) return ORC_E_ARG;
  if (p->gpus_per_host < 1 || p->gpus_per_host > 8) return ORC_E_ARG;
  if (p->migration_delay_ms < 0 || p->boot_delay_ms < 0 || p->retry_interval_ms < 1) return ORC_E_ARG;
  if (p->max_retries < 0 || p->max_retries > 15) return ORC_E_ARG;
  if (p->cap_milli < 1 || p->cap_milli > 100000) return ORC_E_ARG;
  if (p->flags & ~(uint32_t)(ORC_F_MIGRATE | ORC_F_SCALE_OUT | ORC_F_SCALE_IN | ORC_F_AUTOSCALE |
                            ORC_F_DYNAMIC_SR | ORC_F_STICKY | ORC_F_WARM_POOL | ORC_F_CLOSED_LOOP)) return ORC_E_ARG;
  if ((p->flags & ORC_F_CLOSED_LOOP) && (p->flags & (ORC_F_SCALE_IN | ORC_F_AUTOSCALE))) return ORC_E_ARG;
  if (p->flags & ORC_F_WARM_POOL) {
    if (p->warm_pool_per_host < 1 || p->warm_pool_per_host > 4) return ORC_E_ARG;
    if (p->warm_migration_delay_ms < 0 || p->prewarm_delay_ms < 0) return ORC_E_ARG;
  }
  if (p->flags & (ORC_F_SCALE_IN | ORC_F_AUTOSCALE)) {
    if (p->scale_interval_ms < 1 || p->min_hosts < 0) return ORC_E_ARG;
  }
  if (p->flags & ORC_F_SCALE_IN) {
    if (p->scale_in_idle_pct < 0 || p->scale_in_idle_pct > 100) return ORC_E_ARG;
  }
  if (p->flags & ORC_F_AUTOSCALE) {
    if (p->autoscale_f_milli < 0 || p->autoscale_f_milli > 100000) return ORC_E_ARG;
    if (p->scaling_buffer_hosts < 0 || p->scaling_buffer_hosts > 1024) return ORC_E_ARG;
  }
  if (n_events < 0 || n_sessions < 0 || n_sessions > 65536) return ORC_E_ARG;
  for (int32_t s = 0; s < n_sessions; s++)
    if (sess_gpus[s] < 1 || sess_gpus[s] > p->gpus_per_host) return ORC_E_INPUT;
  int32_t prev = 0;
  for (int64_t i = 0; i < n_events; i++) {
    int kind = (int)((uint32_t)ev_sk[i] >> 24), s = ev_sk[i] & 0xFFFFFF;
    if (ev_time[i] < prev) return ORC_E_INPUT;
    prev = ev_time[i];
    if (kind > ORC_EV_END || s >= n_sessions) return ORC_E_INPUT;
    if (kind == ORC_EV_CELL && (ev_dur[i] < 1 || ev_dur[i] > MAX_DUR)) return ORC_E_INPUT;
  }
  int64_t slowest = p->migration_delay_ms;
  if ((p->flags & ORC_F_WARM_POOL) && p->warm_migration_delay_ms > slowest) slowest = p->warm_migration_delay_ms;
  int64_t horizon = (int64_t)prev + MAX_DUR + (int64_t)p->max_retries * p->retry_interval_ms +
                    p->boot_delay_ms + slowest + ((p->flags & ORC_F_WARM_POOL) ? p->prewarm_delay_ms : 0) +
                    /* the next auto-scaler period is pushed one interval past the timer that ran */
                    ((p->flags & (ORC_F_SCALE_IN | ORC_F_AUTOSCALE)) ? p->scale_interval_ms : 0);
  if (horizon >= 2147483647LL) return ORC_E_INPUT;
  return 0;
}

int orc_replay(const orc_params *p,
               int64_t n_events, const int32_t *ev_time, const int32_t *ev_dur,
               const int32_t *ev_sk,
               int32_t n_sessions, const uint8_t *sess_gpus,
               orc_result *out, uint64_t *log, int64_t log_cap, orc_final *fin) {
  if (!p || !out) return ORC_E_ARG;
  int v = validate(p, n_events, ev_time, ev_dur, ev_sk, n_sessions, sess_gpus);
  if (v) return v;

  sim m;
  memset(&m, 0, sizeof m);
  m.p = p; m.H = p->hosts_max; m.G = p->gpus_per_host;
  m.n_sess = n_sessions;
  m.log = log; m.log_cap = log ? log_cap : 0;
  m.hosts = (host_rec *)calloc((size_t)m.H, sizeof(host_rec));
  m.sess = (sess_rec *)calloc((size_t)(n_sessions > 0 ? n_sessions : 1), sizeof(sess_rec));
  m.cap_heap = 64;
  m.heap = (tmr *)malloc((size_t)m.cap_heap * sizeof(tmr));
  if (!m.hosts || !m.sess || !m.heap) { free(m.hosts); free(m.sess); free(m.heap); return ORC_E_NOMEM; }

  for (int h = 0; h < p->hosts_initial; h++) m.hosts[h].state = H_READY;
  m.n_on = p->hosts_initial;
  m.r.peak_hosts = (uint32_t)m.n_on;
  for (int s = 0; s < n_sessions; s++) {
    m.sess[s].g = sess_gpus[s];
    m.sess[s].last_exec = -1;
    m.sess[s].exec_slot = -1;
  }
  m.r.digest = 0xCBF29CE484222325ULL;
  if (p->flags & (ORC_F_SCALE_IN | ORC_F_AUTOSCALE)) heap_push(&m, p->scale_interval_ms, T_TICK, 0);
  const int closed = (p->flags & ORC_F_CLOSED_LOOP) != 0;
  char *first_start = NULL;
  if (closed) {
    /* chain every session's events: first START, then its CELLs up to and including its first END */
    size_t ne = (size_t)(n_events > 0 ? n_events : 1), ns = (size_t)(n_sessions > 0 ? n_sessions : 1);
    m.ev_dur = ev_dur; m.ev_sk = ev_sk;
    m.think = (int32_t *)calloc(ne, sizeof(int32_t));
    m.next_ev = (int64_t *)malloc(ne * sizeof(int64_t));
    m.cursor = (int64_t *)malloc(ns * sizeof(int64_t));
    first_start = (char *)calloc(ne, 1);
    int64_t *last = (int64_t *)malloc(ns * sizeof(int64_t));       /* last chained event of the session */
    int32_t *anchor = (int32_t *)calloc(ns, sizeof(int32_t));      /* its nominal end                   */
    char *closed_s = (char *)calloc(ns, 1);                        /* the session's END has been seen   */
    if (!m.think || !m.next_ev || !m.cursor || !first_start || !last || !anchor || !closed_s) m.err = ORC_E_NOMEM;
    for (int s = 0; s < n_sessions && !m.err; s++) { m.cursor[s] = -1; last[s] = -1; }
    for (int64_t i = 0; i < n_events && !m.err; i++) {
      int kind = (int)((uint32_t)ev_sk[i] >> 24), s = ev_sk[i] & 0xFFFFFF;
      m.next_ev[i] = -1;
      if (kind == ORC_EV_START) {
        if (last[s] < 0) { first_start[i] = 1; last[s] = i; anchor[s] = ev_time[i]; }
        continue;
      }
      if (last[s] < 0 || closed_s[s]) continue;
      m.think[i] = ev_time[i] > anchor[s] ? ev_time[i] - anchor[s] : 0;
      if (first_start[last[s]]) m.cursor[s] = i; else m.next_ev[last[s]] = i;
      last[s] = i;
      anchor[s] = kind == ORC_EV_CELL ? ev_time[i] + ev_dur[i] : ev_time[i];
      if (kind == ORC_EV_END) closed_s[s] = 1;
    }
    free(last); free(anchor); free(closed_s);
  }

  /* arrivals in input order; every timer due at or before an arrival runs first */
  for (int64_t i = 0; i < n_events && !m.err; i++) {
    int32_t t = ev_time[i];
    if (closed && !first_start[i]) continue;        /* everything else comes by its session's chain */
    while (m.n_heap > 0 && m.heap[0].time <= t && !m.err) run_timer(&m, heap_pop(&m));
    if (m.err) break;
    advance(&m, t);
    int kind = (int)((uint32_t)ev_sk[i] >> 24), s = ev_sk[i] & 0xFFFFFF;
    if (kind == ORC_EV_START) on_session_start(&m, s);
    else if (kind == ORC_EV_CELL) on_cell(&m, s, ev_dur[i]);
    else on_session_end(&m, s);
    if (p->check && !m.err) verify(&m);
  }
  /* drain: a TICK runs only while some other timer is still pending */
  while (m.n_heap > 0 && !m.err) {
    if (m.heap[0].prio == T_TICK && m.n_heap == 1) break;
    run_timer(&m, heap_pop(&m));
  }

  /* the session lifetimes a Reservation policy would hold GPUs for (the paper's "Baselines" section) */
  m.r.t_end_ms = m.clock;
  for (int s = 0; s < n_sessions; s++) {
    const sess_rec *q = &m.sess[s];
    if (q->state == S_UNPLACED || q->state == S_REJECTED) continue;
    int32_t end = q->has_end ? q->end_time : m.clock;
    m.r.reservation_gpu_ms += (int64_t)q->g * ((int64_t)end - q->t_placed);
  }

  if (p->check && !m.err) {
    uint32_t hs = 0;
    for (int b = 0; b < 32; b++) hs += m.r.delay_hist[b];
    if (m.chk_commit_integral != m.r.gpu_ms_committed) m.err = ORC_E_INVARIANT - 8;
    else if (m.r.cells_total != m.r.cells_started + m.r.cells_aborted +
                                m.r.cells_dropped_busy + m.r.cells_dropped_unplaced)
      m.err = ORC_E_INVARIANT - 9;
    else if (hs != m.r.cells_started) m.err = ORC_E_INVARIANT - 10;
    else if (m.r.gpu_ms_committed - m.r.gpu_ms_executed != m.chk_wait_gpu_ms) m.err = ORC_E_INVARIANT - 11;
    else if (m.sum_C != 0) m.err = ORC_E_INVARIANT - 12;
  }

  if (fin && !m.err) {
    for (int h = 0; h < m.H; h++) {
      if (fin->host_state) fin->host_state[h] = m.hosts[h].state;
      if (fin->host_committed) fin->host_committed[h] = m.hosts[h].C;
      if (fin->host_subscribed) fin->host_subscribed[h] = m.hosts[h].S;
      if (fin->host_nrep) fin->host_nrep[h] = m.hosts[h].nrep;
    }
    for (int s = 0; s < n_sessions; s++) {
      if (fin->sess_state) fin->sess_state[s] = m.sess[s].state;
      if (fin->sess_hosts)
        for (int i = 0; i < R; i++)
          fin->sess_hosts[s * R + i] =
              (m.sess[s].state == S_UNPLACED || m.sess[s].state == S_REJECTED) ? -1 : m.sess[s].host[i];
    }
  }
  *out = m.r;
  int err = m.err;
  free(m.hosts); free(m.sess); free(m.heap);
  free(m.think); free(m.next_ev); free(m.cursor); free(first_start);
  return err;
}

int orc_sizeof_result(void) { return (int)sizeof(orc_result); }

/* ---- "Monetary Cost" section: billing ------------------------------------------------------ */
static int64_t ratio(int64_t amount, int64_t num, int64_t den) {
  return (int64_t)((unsigned __int128)amount * (unsigned __int128)num / (unsigned __int128)den);
}

void orc_billing(const orc_result *r, int G, int64_t price, int markup_pct, int standby_permille,
                 orc_bill *out) {
  const int64_t ms_per_hour = 3600000;
  /* time replicas spent executing: every started cell runs for its duration */
  int64_t exec_ms = r->sum_tct_ms - r->sum_delay_ms;
  int64_t standby_ms = r->replica_ms - exec_ms;
  if (standby_ms < 0) standby_ms = 0;             /* no replicas (Batch baseline): nothing stands by */
  /* host-hours = GPU-ms / (G * ms per hour) */
  out->provider_cost = ratio(r->gpu_ms_provisioned, price, (int64_t)G * ms_per_hour);
  out->usage_revenue = ratio(r->gpu_ms_executed, price * markup_pct, (int64_t)G * ms_per_hour * 100);
  out->standby_revenue = ratio(standby_ms, price * markup_pct * standby_permille, ms_per_hour * 100 * 1000);
  out->reservation_revenue = ratio(r->reservation_gpu_ms, price * markup_pct, (int64_t)G * ms_per_hour * 100);
}
