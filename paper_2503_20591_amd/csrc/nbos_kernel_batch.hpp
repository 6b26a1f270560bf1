// nbos_kernel_batch.hpp — replay of the Batch baseline (the paper's "Baselines" section): every cell is a job of its
// own, first come first served, a container per job. One workgroup (one wave64) per replay, any cluster
// size up to NBOS_MAX_HOSTS.
//
// LDS per replay
//   fin[h][8]    per-GPU "busy until" times, one 32-byte row per host, kept sorted ascending (slots
//                beyond G hold NEVER): a GPU is held at time t iff fin > t, the host has g idle GPUs
//                from fin[g-1] on, and an allocation rewrites the row in one step (the g smallest
//                entries leave, g copies of the finish time enter at their sorted place).
//                Completions need no timer (see below).
//   ready_at[h]  0 for initial hosts, NEVER while off, boot completion time while provisioning.
//   sess[s]      12 bytes: busy-until time of the session's job, or its submit time while it waits in the
//                queue; its duration; g and a "waiting" bit.
//   fifo         ring of waiting jobs (16-bit session ids); at most one per session.
//
// The CPU reference runs completions and "host ready" as timers and looks at the queue after each
// instant. Here nothing is queued as a timer. The job at the head of the queue first meets the scheduler
// at T0 = max(its submit time, the time the previous head got its GPUs). If some ready host has g idle
// GPUs at T0 it starts there. Otherwise nothing is allocated until it starts (it blocks the queue), so
// the busy-until times do not change while it waits and the instant it starts is known in closed form:
// E = min over hosts of max(ready_at, g-th smallest busy-until time of the host), which is the time of a
// completion or of a host turning ready, i.e. an instant at which the reference serves the queue.
// A GPU with fin <= E is free at E exactly when the reference has applied every completion of that
// instant. The queue is advanced up to the time of each arriving event before the event is looked at
// (timers due at or before an arrival run before it), and to the end after the last one.
#pragma once
#include "nbos_common.hpp"

namespace {
namespace batchk {

enum { CS_QUEUED, CS_SO, CS_PEAK, CS_NON, CS_MAXDELAY, CS_N32 };
enum { CL_SUMDELAY, CL_PROV, CL_N64 };

struct SessRec { int32_t time, dur, gq; };      // gq = g | waiting << 8
constexpr int32_t WAITING = 1 << 8;

struct Lds {
  unsigned long long *c64;
  uint32_t *c32, *hist;
  int4 *fin;
  int32_t *ready_at;
  int32_t *cmy, *cmh;           // [8][NCH] per request size and chunk of 64 hosts: see chunk_min_rescan
  SessRec *sess;
  uint16_t *fifo;
};
constexpr int NCH = NBOS_MAX_HOSTS / WAVE;

struct State {
  uint32_t n_dec, c_total, c_started, c_imm, c_busy;
  int64_t sum_dur, g_exec, g_hold;
  uint64_t digest;
  int32_t q_head, q_n;          // ring: index of the head, jobs waiting
  int32_t last_T;               // when the previous head got its GPUs
  int32_t head_E;               // start time worked out for a waiting head, or -1
  bool head_asked;              // the waiting head has asked for a host
  int32_t lazy_max, t_end;
  int32_t status;               // NBOS_OK, or NBOS_E_RANGE once a time leaves the int32 range
};

struct Ctx {
  const KParams &p;
  Lds m;
  int lane;
  int ring;                     // ring capacity
  uint64_t *dlog;
};

__device__ __forceinline__ void decide(Ctx &c, State &r, int32_t now, uint32_t outcome, uint32_t s, uint32_t host) {
  const uint64_t code = (uint64_t)host | ((uint64_t)outcome << 12) | ((uint64_t)s << 16) | ((uint64_t)(uint32_t)now << 32);
  r.digest = r.digest * DIGEST_PRIME + code;
  if (c.dlog) {
    if (c.lane == 0 && (int64_t)r.n_dec < c.p.dlog_stride) c.dlog[r.n_dec] = code;
  }
  r.n_dec++;
}

// GPUs of host h held at time `now` (the slots beyond G hold NEVER and are taken off again)
__device__ __forceinline__ int committed(const Ctx &c, int h, int32_t now) {
  const int4 a = c.m.fin[2 * h], b = c.m.fin[2 * h + 1];
  return (a.x > now) + (a.y > now) + (a.z > now) + (a.w > now) + (b.x > now) + (b.y > now) + (b.z > now) + (b.w > now) -
         (NGPU - c.p.G);
}

// ---- per chunk of 64 hosts and request size g: the earliest time one of its hosts has g GPUs idle ----------
// y_h(g) = max(ready_at, g-th smallest busy-until time) = max(ready_at, fin[g-1]) (the rows are kept sorted):
// host h can take a job of g GPUs from y_h(g) on, if nothing new is allocated on it. cmy[g-1][chunk] is the
// minimum of y_h(g) over the chunk's hosts and cmh the host it sits on (the lowest such host). A job's scan
// then only looks at the chunks whose minimum is not later than its time, and the earliest time any host
// can take it is the minimum over at most 16 values. y_h only changes when GPUs of h are allocated (it
// grows: the minimum of h's chunk moves only if it sat on h) or when h is provisioned (it drops to ready_at).
__device__ __forceinline__ void chunk_min_rescan(const Ctx &c, int ch, int gi) {
  const int h = ch * WAVE + c.lane;
  const int32_t *row = (const int32_t *)&c.m.fin[2 * h];
  const int32_t ra = c.m.ready_at[h];
  const int32_t f = row[gi];
  const int32_t y = f > ra ? f : ra;
  const int32_t mn = (int32_t)wave_min((uint32_t)y);
  const int at = (int)__builtin_ctzll(wballot(y == mn));
  if (c.lane == 0) { c.m.cmy[gi * NCH + ch] = mn; c.m.cmh[gi * NCH + ch] = ch * WAVE + at; }
}

// GPUs of host h have just been allocated: the minima that sat on h are worked out again (lane g-1 looks)
__device__ __forceinline__ void chunk_min_host_bound(const Ctx &c, int h) {
  if (c.p.HP == WAVE) return;                    // one chunk: the scans look at every host anyway
  wave_sync();
  const int ch = h >> 6;
  const bool hit = c.lane < NGPU && c.m.cmh[c.lane * NCH + ch] == h;
  for (uint64_t w = wballot(hit); w != 0; w &= w - 1) chunk_min_rescan(c, ch, (int)__builtin_ctzll(w));
}

// host h has just been provisioned, ready at ra, all its GPUs idle
__device__ __forceinline__ void chunk_min_host_added(const Ctx &c, int h, int32_t ra) {
  if (c.p.HP == WAVE) return;
  wave_sync();
  const int ch = h >> 6;
  if (c.lane < c.p.G) {
    const int at = c.lane * NCH + ch;
    const int32_t mn = c.m.cmy[at];
    if (ra < mn || (ra == mn && h < c.m.cmh[at])) { c.m.cmy[at] = ra; c.m.cmh[at] = h; }
  }
}

// ready host with the fewest GPUs held at time T that has g idle ones; ties to the lowest index.
// Returns committed << 10 | host, or 0xFFFFFFFF; then `earliest` is the earliest time at which some host
// that is on has g idle GPUs if nothing new is allocated.
__device__ __forceinline__ uint32_t best_host(const Ctx &c, int32_t T, int g, int32_t &earliest) {
  wave_sync();
  if (c.p.HP == WAVE) {
    // one chunk: lane = host, both answers from one look
    const int32_t *row = (const int32_t *)&c.m.fin[2 * c.lane];
    const int32_t ra = c.m.ready_at[c.lane];
    const int32_t free_at = row[g - 1];
    const int32_t y = free_at > ra ? free_at : ra;
    uint32_t best = 0xFFFFFFFFu;
    if (wballot(y <= T) != 0) {
      const int C = committed(c, c.lane, T);
      if (y <= T) best = ((uint32_t)C << 10) | (uint32_t)c.lane;
    }
    const uint32_t key = wave_min(best);
    earliest = key == 0xFFFFFFFFu ? (int32_t)wave_min((uint32_t)y) : T;
    return key;
  }
  const int32_t mine = c.lane < c.p.HP / WAVE ? c.m.cmy[(g - 1) * NCH + c.lane] : NEVER;
  uint64_t chunks = wballot(mine <= T);            // the chunks in which somebody can take the job at T
  if (chunks == 0) { earliest = (int32_t)wave_min((uint32_t)mine); return 0xFFFFFFFFu; }
  uint32_t best = 0xFFFFFFFFu;
  for (; chunks != 0; chunks &= chunks - 1) {
    const int h = (int)__builtin_ctzll(chunks) * WAVE + c.lane;
    const int32_t *row = (const int32_t *)&c.m.fin[2 * h];
    const int32_t ra = c.m.ready_at[h];
    const int32_t free_at = row[g - 1];
    const bool ok = ra <= T && free_at <= T;
    const int C = committed(c, h, T);
    if (ok) best = umin(best, ((uint32_t)C << 10) | (uint32_t)h);
  }
  earliest = T;
  return wave_min(best);
}

// Serve the queue up to time `until`: the head gets its GPUs as soon as a host can give them.
__device__ __forceinline__ void serve_queue(Ctx &c, State &r, int32_t until) {
  while (r.q_n > 0 && r.status == NBOS_OK) {
    wave_sync();
    const int32_t s = uni((int32_t)c.m.fifo[r.q_head]);
    const SessRec j = c.m.sess[s];
    const int32_t t_submit = uni(j.time), dur = uni(j.dur);
    const int g = uni(j.gq) & 0xFF;
    int32_t T = t_submit > r.last_T ? t_submit : r.last_T;          // the head meets the scheduler
    if (T > until) break;
    uint32_t key = 0xFFFFFFFFu;
    int32_t first_free = NEVER;
    if (r.head_E < 0) {
      key = best_host(c, T, g, first_free);
      if (key == 0xFFFFFFFFu) {
        // nothing at T: ask for one more host (once), then the start time is a closed form
        if ((c.p.flags & NBOS_F_SCALE_OUT) && !r.head_asked) {
          wave_sync();
          const int n_on = (int)uni(c.m.c32[CS_NON]);
          if (n_on < c.p.Hmax) {
            int h = 0;
            for (int base = 0; base < c.p.HP; base += WAVE) {
              const int hh = base + c.lane;
              const uint64_t off = wballot(hh < c.p.Hmax && c.m.ready_at[hh] == NEVER);
              if (off) { h = base + (int)__builtin_ctzll(off); break; }
            }
            if ((int64_t)T + c.p.boot >= 0x7FFFFFFFLL) { r.status = NBOS_E_RANGE; break; }
            const int32_t ra = T + c.p.boot;
            if (c.lane == 0) {
              c.m.ready_at[h] = ra;
              atomicAdd(&c.m.c32[CS_NON], 1u);
              atomicAdd(&c.m.c32[CS_SO], 1u);
              atomicMax(&c.m.c32[CS_PEAK], (uint32_t)(n_on + 1));
              atomicAdd(&c.m.c64[CL_PROV], (unsigned long long)(-(int64_t)c.p.G * T));
            }
            r.lazy_max = r.lazy_max > ra ? r.lazy_max : ra;
            decide(c, r, T, NBOS_D_BATCH_HOST, (uint32_t)s, (uint32_t)h);
            first_free = first_free < ra ? first_free : ra;     // the new host has all its GPUs idle once it is up
            chunk_min_host_added(c, h, ra);
          }
          r.head_asked = true;
        }
        r.head_E = first_free;
      }
    }
    if (key == 0xFFFFFFFFu) {
      if (r.head_E > until) break;                  // still waiting when the next event arrives
      T = r.head_E;
      int32_t unused;
      key = best_host(c, T, g, unused);
    }
    // a long queue can push a job beyond the int32 time range: the replay ends as invalid
    if ((int64_t)T + c.p.batch_delay + dur >= 0x7FFFFFFFLL) { r.status = NBOS_E_RANGE; break; }
    // the job gets its GPUs at T on host h: container start, then the cell
    const int h = (int)(key & 1023u);
    const int32_t start = T + c.p.batch_delay, finish = start + dur;
    const int32_t delay = start - t_submit;
    wave_sync();
    {
      // the g GPUs that have been free longest (entries 0..g-1, all <= T) are taken until `finish`:
      // entries g.. that are <= finish move down g places, then g copies of finish, the rest stays
      int32_t *row = (int32_t *)&c.m.fin[2 * h];
      const int k = c.lane & 7;
      const int32_t own = row[k];
      const int32_t up = row[(k + g) & 7];
      const int m = __builtin_popcountll(wballot(c.lane < 8 && k >= g && own <= finish));
      const int32_t nv = k < m ? up : (k < m + g ? finish : own);
      wave_sync();
      if (c.lane < 8) row[k] = nv;
    }
    chunk_min_host_bound(c, h);
    int b = delay == 0 ? 0 : 32 - __builtin_clz((uint32_t)delay);
    b = b > 31 ? 31 : b;
    if (c.lane == 0) {
      c.m.sess[s].time = finish; c.m.sess[s].gq = g;
      atomicAdd(&c.m.hist[b], 1u);
      atomicAdd(&c.m.c64[CL_SUMDELAY], (unsigned long long)delay);
      atomicMax(&c.m.c32[CS_MAXDELAY], (uint32_t)delay);
      if (T != t_submit) atomicAdd(&c.m.c32[CS_QUEUED], 1u);
    }
    r.c_started++;
    if (T == t_submit) r.c_imm++;
    r.sum_dur += dur;
    r.g_exec += (int64_t)g * dur;
    r.g_hold += (int64_t)g * (finish - T);
    r.lazy_max = r.lazy_max > finish ? r.lazy_max : finish;
    decide(c, r, T, NBOS_D_BATCH_START, (uint32_t)s, (uint32_t)h);
    r.last_T = T;
    r.head_E = -1;
    r.head_asked = false;
    r.q_head = r.q_head + 1 == c.ring ? 0 : r.q_head + 1;
    r.q_n--;
  }
}

__global__ void __launch_bounds__(WAVE) nbos_replay_batch_kernel(KParams p) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int rep = launch_slot_replay(p);
  const int lane = threadIdx.x;
  if (rep >= p.n_replays) return;

  const int trace = p.trace_of_replay[rep];
  const int64_t ev_lo = p.ev_offset[trace], ev_hi = p.ev_offset[trace + 1];
  const int s_lo = p.sess_offset[trace];
  const int n_sess = p.sess_offset[trace + 1] - s_lo;

  Lds m;
  unsigned char *q = lds_raw;
  m.c64 = (unsigned long long *)q;  q += 8 * 8;
  m.c32 = (uint32_t *)q;            q += 16 * 4;
  m.hist = (uint32_t *)q;           q += 32 * 4;
  m.fin = (int4 *)q;                q += (size_t)p.HP * 32;
  m.ready_at = (int32_t *)q;        q += (size_t)p.HP * 4;
  m.cmy = (int32_t *)q;             q += NGPU * NCH * 4;
  m.cmh = (int32_t *)q;             q += NGPU * NCH * 4;
  m.sess = (SessRec *)q;            q += (size_t)p.n_cap * 12;
  m.fifo = (uint16_t *)q;

  if (lane < 8) m.c64[lane] = 0;
  if (lane < 16) m.c32[lane] = lane == CS_NON || lane == CS_PEAK ? (uint32_t)p.H0 : 0u;
  if (lane < 32) m.hist[lane] = 0;
  for (int i = lane; i < 8 * p.HP; i += WAVE) ((int32_t *)m.fin)[i] = (i & 7) < p.G ? 0 : NEVER;
  for (int h = lane; h < p.HP; h += WAVE) m.ready_at[h] = h < p.H0 ? 0 : NEVER;
  for (int s = lane; s < n_sess; s += WAVE) { m.sess[s].time = 0; m.sess[s].dur = 0; m.sess[s].gq = p.sess_gpus[s_lo + s]; }
  __syncthreads();

  Ctx c{p, m, lane, p.n_cap + 1, p.dlog ? p.dlog + (int64_t)rep * p.dlog_stride : nullptr};
  if (p.HP > WAVE) {
    for (int ch = 0; ch < p.HP / WAVE; ch++)
      for (int gi = 0; gi < NGPU; gi++) chunk_min_rescan(c, ch, gi);
  }
  State r;
  memset(&r, 0, sizeof r);
  r.digest = 0xCBF29CE484222325ULL;
  r.head_E = -1;

  // the events: one per lane per tile, next tile in flight
  int64_t base = ev_lo;
  int32_t vt = 0, vd = 0, vs = 0, nt = 0, nd = 0, ns = 0;
  if (base + lane < ev_hi) { nt = p.ev_time[base + lane]; nd = p.ev_dur[base + lane]; ns = p.ev_sk[base + lane]; }
  while (base < ev_hi && r.status == NBOS_OK) {
    vt = nt; vd = nd; vs = ns;
    const int64_t cur = base;
    base += WAVE;
    if (base + lane < ev_hi) { nt = p.ev_time[base + lane]; nd = p.ev_dur[base + lane]; ns = p.ev_sk[base + lane]; }
    const bool valid = cur + lane < ev_hi;
    const bool is_cell = valid && ((uint32_t)vs >> 24) == NBOS_EV_CELL;
    uint64_t todo = wballot(is_cell);
    r.c_total += (uint32_t)__builtin_popcountll(todo);
    if (ev_hi - cur <= WAVE) {
      const int32_t tl = lane_get(vt, (int)(ev_hi - cur - 1));
      r.t_end = r.t_end > tl ? r.t_end : tl;
    }
    while (todo != 0 && r.status == NBOS_OK) {
      const int i = (int)__builtin_ctzll(todo);
      todo &= todo - 1;
      const int32_t t = lane_get(vt, i), dur = lane_get(vd, i);
      const int32_t s = (int32_t)((uint32_t)lane_get(vs, i) & 0xFFFFFFu);
      serve_queue(c, r, t);                       // everything due at or before the arrival comes first
      wave_sync();
      const SessRec rec = m.sess[s];
      const int32_t gq = uni(rec.gq);
      if ((gq & WAITING) || uni(rec.time) > t) { r.c_busy++; continue; }     // previous job not finished
      int tail = r.q_head + r.q_n;
      tail = tail >= c.ring ? tail - c.ring : tail;
      if (lane == 0) { m.fifo[tail] = (uint16_t)s; m.sess[s].time = t; m.sess[s].dur = dur; m.sess[s].gq = gq | WAITING; }
      r.q_n++;
      serve_queue(c, r, t);
    }
  }
  serve_queue(c, r, NEVER);

  __syncthreads();
  const int32_t t_end = r.t_end > r.lazy_max ? r.t_end : r.lazy_max;
  nbos_stats *out = p.stats + rep;
  if (lane < 32) out->delay_hist[lane] = m.hist[lane];
  if (lane == 0) {
    const int64_t sum_delay = (int64_t)m.c64[CL_SUMDELAY];
    out->status = r.status; out->n_decisions = r.n_dec;
    out->sessions_placed = 0; out->sessions_rejected = 0;
    out->cells_total = r.c_total; out->cells_immediate = r.c_imm; out->cells_started = r.c_started;
    out->cells_queued = m.c32[CS_QUEUED]; out->cells_aborted = 0;
    out->cells_dropped_busy = r.c_busy; out->cells_dropped_unplaced = 0;
    out->executor_reused = 0; out->migrations = 0;
    out->scale_out_hosts = m.c32[CS_SO]; out->scale_in_hosts = 0; out->peak_hosts = m.c32[CS_PEAK];
    out->migrations_warm = 0;
    out->max_delay_ms = (int32_t)m.c32[CS_MAXDELAY]; out->t_end_ms = t_end;
    out->sum_delay_ms = sum_delay; out->sum_tct_ms = r.sum_dur + sum_delay;
    out->gpu_ms_executed = r.g_exec; out->gpu_ms_committed = r.g_hold;
    out->gpu_ms_provisioned = (int64_t)m.c64[CL_PROV] + (int64_t)m.c32[CS_NON] * p.G * t_end;
    out->reservation_gpu_ms = 0; out->sub_gpu_ms = 0; out->replica_ms = 0;
    out->digest = r.digest;
  }
}

}  // namespace batchk
}  // namespace
