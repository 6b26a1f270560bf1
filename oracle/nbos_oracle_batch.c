/*
 * nbos_oracle_batch.c — CPU oracle of the Batch baseline policy.
 *
 * TEST INFRASTRUCTURE (see nbos_oracle.h). Plain C99, single-threaded, eager
 * discrete-event loop with one heap of timers.
 *
 * What it follows: the "Batch" baseline of the paper's "Baselines" section: no long-running
 * kernel, no replicas. Every cell submission is a job of its own: a container is
 * provisioned for it on a server with enough idle GPUs, serves the request and
 * terminates. Jobs are served first come, first served (strict: a job never
 * overtakes an earlier one). Metrics as in sections "Resource Usage & Efficiency", "Interactivity" and "Task Completion Time".
 *
 * Readings taken where the paper leaves a choice open (all deterministic):
 *   - a job holds its g GPUs from the moment they are allocated: for the
 *     container start (batch_start_delay_ms) and then for the cell's duration;
 *     the interactivity delay is queueing time + container start.
 *   - the server is the ready one with the fewest committed GPUs that has g idle
 *     ones, ties to the lowest index.
 *   - the queue is examined after the arrival of a job and after all timers of
 *     one instant (completions, servers turning ready) have been applied.
 *   - with ORC_F_SCALE_OUT a job at the head of the queue that finds no server
 *     asks for one more server, once (ready after boot_delay_ms; Section 3.4.2).
 *   - a cell that arrives while the session's previous job has not finished is
 *     dropped and counted, as in the NotebookOS replay (one cell at a time per
 *     session). SESSION_START / SESSION_END events carry no meaning here.
 *   - timers due at or before an arrival run before it; at one instant
 *     completions run before servers turn ready.
 *   - times are int32 milliseconds: a replay whose queue pushes a job to 2^31 - 1 or
 *     beyond ends with ORC_E_INPUT.
 */
#include "nbos_oracle.h"
#include <stdlib.h>
#include <string.h>

#define MAX_DUR 86400000

enum { H_OFF = 0, H_BOOT = 1, H_READY = 2 };
enum { J_IDLE = 0, J_QUEUED = 1, J_RUNNING = 2 };
enum { T_COMPLETE = 0, T_HOST_READY = 1 };

typedef struct { int32_t time; int32_t prio; int32_t id; } tmr;
typedef struct { int state; int32_t ready_at; int C; } host_rec;
typedef struct { int state, g, host, asked; int32_t t_submit, dur; } job_rec;   /* one per session */

typedef struct {
  const orc_params *p;
  int H, G, n_on;
  host_rec *hosts;
  job_rec *job;
  int n_sess;
  int *fifo; int head, count;          /* ring of session ids, capacity n_sess + 1 */
  tmr *heap; int n_heap, cap_heap;
  int32_t clock;
  orc_result r;
  uint64_t *log; int64_t log_cap;
  int err;
} sim;

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

static void decide(sim *m, int outcome, int s, int host) {
  uint64_t code = (uint64_t)(uint32_t)host | ((uint64_t)outcome << 12) | ((uint64_t)s << 16) |
                  ((uint64_t)(uint32_t)m->clock << 32);
  m->r.digest = m->r.digest * 0x100000001B3ULL + code;
  if (m->log && (int64_t)m->r.n_decisions < m->log_cap) m->log[m->r.n_decisions] = code;
  m->r.n_decisions++;
}

static void advance(sim *m, int32_t t) {
  m->r.gpu_ms_provisioned += (int64_t)m->n_on * m->G * ((int64_t)t - m->clock);
  m->clock = t;
}

/* Serve the queue in order for as long as its head finds a server. */
static void dispatch(sim *m) {
  while (m->count > 0) {
    int s = m->fifo[m->head];
    job_rec *j = &m->job[s];
    int best = -1;
    for (int h = 0; h < m->H; h++) {
      const host_rec *x = &m->hosts[h];
      if (x->state != H_READY || m->G - x->C < j->g) continue;
      if (best < 0 || x->C < m->hosts[best].C) best = h;      /* ties stay with the lower index */
    }
    if (best < 0) {
      if ((m->p->flags & ORC_F_SCALE_OUT) && !j->asked && m->n_on < m->H) {
        for (int h = 0; h < m->H; h++)
          if (m->hosts[h].state == H_OFF) {
            if ((int64_t)m->clock + m->p->boot_delay_ms >= 2147483647LL) { m->err = ORC_E_INPUT; return; }
            m->hosts[h].state = H_BOOT;
            m->hosts[h].ready_at = m->clock + m->p->boot_delay_ms;
            heap_push(m, m->hosts[h].ready_at, T_HOST_READY, h);
            m->n_on++;
            if ((uint32_t)m->n_on > m->r.peak_hosts) m->r.peak_hosts = (uint32_t)m->n_on;
            m->r.scale_out_hosts++;
            decide(m, ORC_D_BATCH_HOST, s, h);
            break;
          }
        j->asked = 1;
      }
      return;
    }
    /* a long queue can push a job beyond the int32 time range: the replay is invalid then */
    if ((int64_t)m->clock + m->p->batch_start_delay_ms + j->dur >= 2147483647LL) { m->err = ORC_E_INPUT; return; }
    /* allocate: the container starts now, the cell runs after the start delay */
    int32_t start = m->clock + m->p->batch_start_delay_ms;
    int32_t finish = start + j->dur;
    int32_t delay = start - j->t_submit;
    m->hosts[best].C += j->g;
    j->state = J_RUNNING; j->host = best;
    heap_push(m, finish, T_COMPLETE, s);
    m->r.cells_started++;
    if (m->clock == j->t_submit) m->r.cells_immediate++; else m->r.cells_queued++;
    m->r.sum_delay_ms += delay;
    if (delay > m->r.max_delay_ms) m->r.max_delay_ms = delay;
    int b = 0;
    for (int32_t x = delay; x > 0; x >>= 1) b++;
    if (b > 31) b = 31;
    m->r.delay_hist[b]++;
    m->r.sum_tct_ms += (int64_t)finish - j->t_submit;
    m->r.gpu_ms_executed += (int64_t)j->g * j->dur;
    m->r.gpu_ms_committed += (int64_t)j->g * ((int64_t)finish - m->clock);
    decide(m, ORC_D_BATCH_START, s, best);
    m->head = (m->head + 1) % (m->n_sess + 1);
    m->count--;
  }
}

/* all timers of the earliest pending instant, then one look at the queue */
static void run_instant(sim *m) {
  int32_t T = m->heap[0].time;
  advance(m, T);
  while (m->n_heap > 0 && m->heap[0].time == T) {
    tmr t = heap_pop(m);
    if (t.prio == T_COMPLETE) {
      job_rec *j = &m->job[t.id];
      m->hosts[j->host].C -= j->g;
      j->state = J_IDLE;
    } else {
      m->hosts[t.id].state = H_READY;
    }
  }
  dispatch(m);
}

int orc_replay_batch(const orc_params *p,
                     int64_t n_events, const int32_t *ev_time, const int32_t *ev_dur,
                     const int32_t *ev_sk,
                     int32_t n_sessions, const uint8_t *sess_gpus,
                     orc_result *out, uint64_t *log, int64_t log_cap) {
  if (!p || !out) return ORC_E_ARG;
  if (p->hosts_initial < 1 || p->hosts_max < p->hosts_initial || p->hosts_max > 1024) return ORC_E_ARG;
  if (p->gpus_per_host < 1 || p->gpus_per_host > 8) return ORC_E_ARG;
  if (p->boot_delay_ms < 0 || p->batch_start_delay_ms < 0 || p->batch_start_delay_ms > MAX_DUR) return ORC_E_ARG;
  if (p->flags & ~(uint32_t)(ORC_F_BATCH | ORC_F_SCALE_OUT)) return ORC_E_ARG;
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

  sim m;
  memset(&m, 0, sizeof m);
  m.p = p; m.H = p->hosts_max; m.G = p->gpus_per_host; m.n_sess = n_sessions;
  m.log = log; m.log_cap = log ? log_cap : 0;
  m.hosts = (host_rec *)calloc((size_t)m.H, sizeof(host_rec));
  m.job = (job_rec *)calloc((size_t)(n_sessions > 0 ? n_sessions : 1), sizeof(job_rec));
  m.fifo = (int *)calloc((size_t)n_sessions + 1, sizeof(int));
  m.cap_heap = 64;
  m.heap = (tmr *)malloc((size_t)m.cap_heap * sizeof(tmr));
  if (!m.hosts || !m.job || !m.fifo || !m.heap) {
    free(m.hosts); free(m.job); free(m.fifo); free(m.heap);
    return ORC_E_NOMEM;
  }
  for (int h = 0; h < p->hosts_initial; h++) m.hosts[h].state = H_READY;
  m.n_on = p->hosts_initial;
  m.r.peak_hosts = (uint32_t)m.n_on;
  for (int s = 0; s < n_sessions; s++) m.job[s].g = sess_gpus[s];
  m.r.digest = 0xCBF29CE484222325ULL;

  for (int64_t i = 0; i < n_events && !m.err; i++) {
    int32_t t = ev_time[i];
    while (m.n_heap > 0 && m.heap[0].time <= t && !m.err) run_instant(&m);
    advance(&m, t);
    int kind = (int)((uint32_t)ev_sk[i] >> 24), s = ev_sk[i] & 0xFFFFFF;
    if (kind != ORC_EV_CELL) continue;
    job_rec *j = &m.job[s];
    m.r.cells_total++;
    if (j->state != J_IDLE) { m.r.cells_dropped_busy++; continue; }
    j->state = J_QUEUED; j->t_submit = t; j->dur = ev_dur[i]; j->asked = 0;
    m.fifo[(m.head + m.count) % (n_sessions + 1)] = s;
    m.count++;
    dispatch(&m);
  }
  while (m.n_heap > 0 && !m.err) run_instant(&m);
  m.r.t_end_ms = m.clock;

  if (p->check && !m.err) {
    /* every job was served and every GPU given back */
    uint32_t hs = 0;
    for (int b = 0; b < 32; b++) hs += m.r.delay_hist[b];
    if (m.count != 0) m.err = ORC_E_INVARIANT - 1;
    for (int h = 0; h < m.H; h++) if (m.hosts[h].C != 0) m.err = ORC_E_INVARIANT - 2;
    if (m.r.cells_total != m.r.cells_started + m.r.cells_dropped_busy) m.err = ORC_E_INVARIANT - 9;
    if (hs != m.r.cells_started) m.err = ORC_E_INVARIANT - 10;
  }
  *out = m.r;
  int err = m.err;
  free(m.hosts); free(m.job); free(m.fifo); free(m.heap);
  return err;
}
