// nbos_kernel_closed.hpp — closed-loop reading of a trace (the paper's section "Interactive Deep Learning Training": users think and edit
// between the cells they submit) on the any-size kernel's state and policy code.
//
// Only a session's first START keeps its time. Every later CELL / END of the session is due one
// think time after the session's previous cell is over (finished or given up; the first one: after
// the placement). The think time is what the trace leaves between the previous event's nominal end
// (its time, plus its duration for a CELL) and the event's own time, at least 0.
//
// nbos_closed_chain_kernel   once per set of traces: per event the next event of its session and the
//                            think time before that one (a session's chain: its first START, then its
//                            CELLs up to and including its first END). One wave per trace walks the
//                            events in order, a tile of 64 per step; "last chained event" and
//                            "nominal end" per session live in LDS.
// nbos_replay_closed_kernel  one wave per replay. Arrivals from the stream are the first STARTs only;
//                            everything else is a timer (kind QK_NEXT, after the retries of the same
//                            instant, by ascending session). A session has at most one timer, so the
//                            timers that do not fit into the 64 sorted registers wait in the session
//                            records (see refill), and no queue can overflow. A timer in the
//                            registers carries the index of its event and, once loaded, the event's
//                            duration, kind and chain record: timers that come in by a refill have
//                            them gathered for all of them at once, timers scheduled straight into
//                            the registers load them together when the first of them gets to the
//                            head (one round trip to device memory). While a timer waits outside the registers the index is kept in
//                            a cursor array in device memory. The due cells at the head of the sorted
//                            timers are started by the any-size kernel's event-parallel rounds, lane =
//                            timer; their sessions' next events are scheduled all at once.
#pragma once
#include "nbos_kernel_lds.hpp"

namespace {
namespace ldsk {

constexpr int32_t CH_NONE = -1, CH_CLOSED = -2;        // last[s]: no START yet / END seen

__global__ void __launch_bounds__(WAVE) nbos_closed_chain_kernel(const int64_t *ev_offset, const int32_t *ev_time,
                                                                 const int32_t *ev_dur, const int32_t *ev_sk,
                                                                 const int32_t *sess_offset, int2 *chain) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int trace = blockIdx.x, lane = threadIdx.x;
  const int64_t lo = ev_offset[trace], hi = ev_offset[trace + 1];
  const int n_sess = sess_offset[trace + 1] - sess_offset[trace];
  // per session: last chained event, its nominal end, the first lane of the current tile that holds it
  int32_t *last = (int32_t *)lds_raw, *anchor = last + n_sess, *mark = anchor + n_sess;
  for (int s = lane; s < n_sess; s += WAVE) { last[s] = CH_NONE; anchor[s] = 0; mark[s] = MARK_FREE; }
  __syncthreads();
  int32_t nt = 0, nd = 0, nsk = 0;              // the next tile, in flight while the current one is linked
  if (lo + lane < hi) { nt = ev_time[lo + lane]; nd = ev_dur[lo + lane]; nsk = ev_sk[lo + lane]; }
  for (int64_t base = lo; base < hi; base += WAVE) {
    const int cnt = hi - base < WAVE ? (int)(hi - base) : WAVE;
    const int32_t idx0 = (int32_t)(base - lo);
    const bool valid = lane < cnt;
    const int32_t t = nt, d = nd;
    const uint32_t sk = (uint32_t)nsk;
    if (base + WAVE + lane < hi) { nt = ev_time[base + WAVE + lane]; nd = ev_dur[base + WAVE + lane]; nsk = ev_sk[base + WAVE + lane]; }
    const uint32_t kind = sk >> 24, s = sk & 0xFFFFFFu;
    int32_t nx = -1, ny = -1;                   // this lane's record; ny = -1: in no chain
    // Sessions are independent, and a tile rarely holds two events of one session: the lanes that are the
    // first of their session in the tile go all at once (their predecessors are in earlier tiles) ...
    if (valid) atomicMin(&mark[s], lane);
    wave_sync();
    const bool first = valid && mark[s] == lane;
    wave_sync();
    if (valid) mark[s] = MARK_FREE;
    if (first) {
      const int32_t L = last[s];
      bool chained = false;
      if (kind == NBOS_EV_START) {
        chained = L == CH_NONE;
      } else if (L >= 0) {
        chained = true;
        const int32_t a = anchor[s];
        chain[lo + L] = make_int2(idx0 + lane, t > a ? t - a : 0);
      }
      if (chained) {
        ny = 0;
        last[s] = kind == NBOS_EV_END ? CH_CLOSED : idx0 + lane;
        anchor[s] = kind == NBOS_EV_CELL ? t + d : t;
      }
    }
    wave_sync();
    // ... the others follow one by one, in trace order
    for (uint64_t w = wballot(valid && !first); w != 0; w &= w - 1) {
      const int i = (int)__builtin_ctzll(w);
      const uint32_t ski = (uint32_t)lane_get((int)sk, i);
      const uint32_t ki = ski >> 24, si = ski & 0xFFFFFFu;
      const int32_t ti = lane_get(t, i), di = lane_get(d, i);
      const int32_t L = last[si];
      bool chained = false;
      if (ki == NBOS_EV_START) {
        chained = L == CH_NONE;
      } else if (L >= 0) {
        chained = true;
        const int32_t a = anchor[si];
        const int32_t th = ti > a ? ti - a : 0;
        if (L >= idx0) { if (lane == L - idx0) { nx = idx0 + i; ny = th; } }     // the predecessor is in this tile
        else if (lane == 0) chain[lo + L] = make_int2(idx0 + i, th);
      }
      wave_sync();
      if (chained) {
        if (lane == i) ny = 0;
        if (lane == 0) {
          last[si] = ki == NBOS_EV_END ? CH_CLOSED : idx0 + i;
          anchor[si] = ki == NBOS_EV_CELL ? ti + di : ti;
        }
      }
      wave_sync();
    }
    if (valid) chain[base + lane] = make_int2(nx, ny);
    // a later tile may overwrite one of these records: wait until the stores have been taken
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  }
}

// The first n sorted timers were cells that an event-parallel round has started (lane i = timer i):
// they leave the registers, and the next event of each of their sessions is scheduled one think time
// after the cell's finish. Those that are not before the earliest timer waiting in the session
// records go there, all at once; the others are inserted into the registers one by one.
template <uint32_t F>
__device__ __forceinline__ void cl_after_round(Ctx<F> &c, Regs &r, int n) {
  const bool succ = c.lane < n && c.qnx >= 0;
  const int32_t ts = succ ? c.qt + (c.qx & 0x0FFFFFFF) + c.qnth : 0;       // in range: checked before the round
  const int32_t es = c.qnx;
  const uint32_t ss = c.qk & 0xFFFFu;
  if (succ) c.cl_cur[ss] = es;
  // drop the n earliest
  const int src = ((c.lane + n) & (WAVE - 1)) << 2;
  c.qt = __builtin_amdgcn_ds_bpermute(src, c.qt);
  c.qk = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)c.qk);
  c.qd = __builtin_amdgcn_ds_bpermute(src, c.qd);
  c.qx = __builtin_amdgcn_ds_bpermute(src, c.qx);
  c.qnx = __builtin_amdgcn_ds_bpermute(src, c.qnx);
  c.qnth = __builtin_amdgcn_ds_bpermute(src, c.qnth);
  r.q_n -= n;
  r.q_head_t = r.q_n > 0 ? lane_get(c.qt, 0) : NEVER;
  const uint32_t ks = (QK_NEXT << 16) | ss;
  const bool far = succ && r.o_n > 0 && !(ts < r.o_min_t || (ts == r.o_min_t && ks < r.o_min_k));
  wave_sync();
  if (far) {
    c.m.sess[ss].z = (int)(((uint32_t)c.m.sess[ss].z & ~(3u << CL_KIND_SHIFT)) | (QK_NEXT << CL_KIND_SHIFT));
    c.m.due[ss] = ts;
  }
  wave_sync();
  r.o_n += __builtin_popcountll(wballot(far));
  for (uint64_t w = wballot(succ && !far); w != 0 && r.status == NBOS_OK; w &= w - 1) {
    const int j = (int)__builtin_ctzll(w);
    timer_push(c, r, lane_get(ts, j), QK_NEXT, (uint32_t)lane_get((int)ss, j), lane_get(es, j));
  }
  if (r.q_n == 0 && r.o_n > 0) {
    refill(c, r);
    r.q_head_t = r.q_n > 0 ? lane_get(c.qt, 0) : NEVER;
  }
}

template <uint32_t F>
__global__ void __launch_bounds__(MAX_WAVES * WAVE) nbos_replay_closed_kernel(KParams p) {
  static_assert(Ctx<F>::closed, "instantiate with a closed-loop flag set");
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int rep = launch_slot_replay(p);
  const int lane = threadIdx.x & (WAVE - 1);
  if (rep >= p.n_replays) return;

  const int trace = p.trace_of_replay[rep];
  const int64_t ev_lo = p.ev_offset[trace], ev_hi = p.ev_offset[trace + 1];
  const int s_lo = p.sess_offset[trace];
  const int n_sess = p.sess_offset[trace + 1] - s_lo;

  const Lds m = lds_carve<true>(p, lds_raw);
  lds_init<true>(p, m, s_lo, n_sess);

  const int32_t caplim = p.cap_milli[rep] * p.G * 3;
  Ctx<F> c{p, m, lane, caplim / 1000, p.dlog ? p.dlog + (int64_t)rep * p.dlog_stride : nullptr,
           NEVER, 0, 0xFFFFFFFFu, 0xFFFFFFFFu, 0, n_sess, p.cl_cursor + (int64_t)rep * p.n_cap,
           p.ev_dur + ev_lo, p.ev_sk + ev_lo, p.cl_chain + ev_lo, 0, -1, 0};
  Regs r;
  memset(&r, 0, sizeof r);
  r.digest = 0xCBF29CE484222325ULL;
  r.q_head_t = NEVER;
  r.o_min_t = NEVER;
  r.min_s = -1;
  r.cl_win = 1024;
  c.nw = (int)(blockDim.x / WAVE);
  c.wid = (int)(threadIdx.x / WAVE);
  c.dyn = dynamic_limit_matters(p, c.flags(), c.slim);
  c.n_on = p.H0;
  if (c.wid != 0) {
    helper_loop(c);
  } else {
  const bool batching = p.batch != 0;
  PROF_BEGIN();
  int cooldown = 0, backoff = 1;            // timers to fire one by one before the next parallel round: doubles
                                            // (up to 64) while rounds start at most one cell, back to 1 when they pay

  bool final = false;
  for (int64_t base = ev_lo; r.status == NBOS_OK; base += WAVE) {
    // S1: of the stream only the first STARTs arrive by themselves (the STARTs that head a chain)
    uint64_t todo = 0;
    int32_t vt = 0, vnx = -1, vnth = -1;
    uint32_t vs = 0;
    if (base < ev_hi) {
      if (base + lane < ev_hi) {
        vt = p.ev_time[base + lane]; vs = (uint32_t)p.ev_sk[base + lane];
        const int2 ch = p.cl_chain[base + lane];
        vnx = ch.x; vnth = ch.y;
      }
      todo = wballot((vs >> 24) == NBOS_EV_START && vnth >= 0);
    } else {
      final = true;
    }
    while (r.status == NBOS_OK) {
      int i = 0;
      int32_t t = NEVER;
      if (todo != 0) { i = (int)__builtin_ctzll(todo); t = lane_get(vt, i); }
      else if (!final) break;
      wave_sync();
      if (r.q_n > 0 && r.q_head_t <= t) {
        if (!(lane_get(c.qx, 0) & CLX_LOADED) && ((uint32_t)lane_get((int)c.qk, 0) >> 16) != QK_END) {
          // the earliest timer was scheduled straight into the registers: its event's duration, kind and
          // chain record are loaded now, and with them those of all other such timers (one round trip)
          if (c.lane < r.q_n && !(c.qx & CLX_LOADED) && (c.qk >> 16) != QK_END) {
            const int2 ch = c.cl_chain[c.qd];
            c.qx = c.cl_dur[c.qd] | (int32_t)(((uint32_t)c.cl_sk[c.qd] >> 24) << 28) | CLX_LOADED;
            c.qnx = ch.x; c.qnth = ch.y;
          }
        }
        // a round needs the next cells of two sessions at the head at least
        if (batching && cooldown == 0 && r.q_n >= 2 && ((uint32_t)lane_get((int)c.qk, 0) >> 16) == QK_NEXT &&
            ((uint32_t)lane_get((int)c.qk, 1) >> 16) == QK_NEXT && lane_get(c.qt, 1) <= t) {
          // ---- event-parallel round over the run of due cells at the head of the sorted timers ----
          // lane i = timer i. A timer can join if it brings the next cell of an idle placed session
          // (its event's data are loaded), and if no successor that the run schedules could come
          // before it: it is earlier than the earliest "finish + think time" over all of them.
          const uint32_t sid = c.qk & 0xFFFFu;
          const bool cell = c.lane < r.q_n && (c.qk >> 16) == QK_NEXT && (c.qx & CLX_LOADED) != 0 &&
                            (((uint32_t)c.qx >> 28) & 3u) == NBOS_EV_CELL && c.qt <= t;
          SessRec rec = {0, 0, 0};
          if (cell) rec = m.sess[sid];
          const int32_t vd = c.qx & 0x0FFFFFFF;
          const int64_t after = (int64_t)c.qt + vd + (c.qnx >= 0 ? c.qnth : 0);
          const bool ok = cell && ((uint32_t)rec.z & 7u) == SS_PLACED && rec.y <= c.qt && !((uint32_t)rec.z & SF_ENDING) &&
                          after < 0x7FFFFFFFLL;
          const int32_t bound = (int32_t)wave_min(ok && c.qnx >= 0 ? (uint32_t)after : 0x7FFFFFFFu);
          const uint64_t out = ~wballot(ok && c.qt < bound);
          const int k = out != 0 ? (int)__builtin_ctzll(out) : WAVE;
          if (k >= 2) {
            const uint64_t run = k >= WAVE ? ~0ull : ((1ull << k) - 1ull);
            bool next_lost;
            PROF(PC_LOOP_ROUND, 1);
            const uint64_t done = batch_round(c, r, run, c.qt, vd, sid, rec, next_lost);
            const int n = __builtin_popcountll(done);
            PROF(PC_ROUND, n);
            if (n <= 1) { cooldown = backoff; backoff = backoff < 64 ? 2 * backoff : 64; }
            else if (n >= 3) backoff = 1;
            if (next_lost && cooldown == 0) cooldown = 1;     // the next timer's cell has just lost its election
            if (n > 0) {
              r.c_total += (uint32_t)n;
              const int32_t tl = lane_get(c.qt, n - 1);
              r.t_end = r.t_end > tl ? r.t_end : tl;
              cl_after_round(c, r, n);
              PROF(PC_TIMER_OTHER, n);           // (closed loop: the started cells' next events are scheduled)
              continue;
            }
          }
        }
        if (cooldown > 0) cooldown--;
        // ---- S2: the earliest timer is due ----
        PROF(PC_LOOP_TIMER, 1);
        const int32_t now = r.q_head_t;
        const uint32_t key = (uint32_t)lane_get((int)c.qk, 0);
        const int32_t e = lane_get(c.qd, 0);
        const int32_t x = lane_get(c.qx, 0), nx = lane_get(c.qnx, 0), nth = lane_get(c.qnth, 0);
        timer_pop(c, r);
        r.t_end = r.t_end > now ? r.t_end : now;
        const uint32_t s = key & 0xFFFFu, kind = key >> 16;
        wave_sync();
        const SessRec cur = m.sess[s];
        const uint32_t hw = uni((uint32_t)cur.x), fl = uni((uint32_t)cur.z);
        const int32_t tm = uni(cur.y);
        if (kind == QK_END) { end_session(c, r, s, hw, fl, now); PROF(PC_END, 1); continue; }
        r.cl_e = e; r.cl_x = x; r.cl_nx = nx; r.cl_nth = nth;
        const int32_t dur = x & 0x0FFFFFFF;
        if (kind == QK_RETRY) {
          PROF(PC_LOOP_ATTEMPT, 1);
          PROF_ATTEMPT_BEGIN(m, r);
          attempt(c, r, s, hw, fl, now, tm, dur);
          PROF_ATTEMPT_END(m, r, true);
        } else if (((uint32_t)x >> 28 & 3u) == NBOS_EV_CELL) {        // the session submits its next cell (S4-S8)
          r.c_total++;
          const uint32_t st = fl & 7u;
          if (st == SS_PLACED && tm <= now && !(fl & SF_ENDING)) {
            PROF(PC_LOOP_ATTEMPT, 1);
            PROF_ATTEMPT_BEGIN(m, r);
            attempt(c, r, s, hw, fl & ~(SF_QONCE | (15u << 8)), now, now, dur);
            PROF_ATTEMPT_END(m, r, false);
          }
          else if (st == SS_PLACED || st == SS_QUEUED) { r.c_busy++; PROF(PC_DROP, 1); }
          else { r.c_unplaced++; PROF(PC_DROP, 1); }
        } else {
          on_session_end(c, r, s, hw, tm, fl, now);     // S9
          PROF(PC_END, 1);
        }
        continue;
      }
      if (todo == 0) break;                 // draining and no timer is left
      todo &= todo - 1;
      const uint32_t s = (uint32_t)lane_get((int)vs, i) & 0xFFFFFFu;
      const uint32_t fl = uni((uint32_t)m.sess[s].z);
      r.t_end = r.t_end > t ? r.t_end : t;
      r.cl_e = (int32_t)(base - ev_lo) + i; r.cl_nx = lane_get(vnx, i); r.cl_nth = lane_get(vnth, i);
      PROF(PC_LOOP_STARTEND, 1);
      session_start(c, r, s, fl, t);        // S3, S7; a placed session's first event is scheduled there
      PROF(PC_START, 1);
    }
    if (final) break;
  }
  wave_sync();
  const int32_t bl = (int32_t)uni(m.c32[CS_BLAZY]);             // finish times bound by the rounds
  r.lazy_max = r.lazy_max > bl ? r.lazy_max : bl;
  helpers_go(c, HC_EXIT, 0, 0, 0);
  }  // wave 0
  write_stats(p, m, r, rep);
  PROF_OUT(rep);
}

}  // namespace ldsk
}  // namespace
