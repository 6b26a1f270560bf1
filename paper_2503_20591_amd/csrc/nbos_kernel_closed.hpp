// nbos_kernel_closed.hpp — closed-loop reading of a trace (paper Section 2.2: users think and edit
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
//                            records (see cl_refill), and no queue can overflow. A timer in the
//                            registers carries the index of its event and, once loaded, the event's
//                            duration, kind and chain record: timers that come in by a refill have
//                            them gathered for all of them at once, a timer scheduled straight into
//                            the registers loads them when it fires (one round trip to device
//                            memory). While a timer waits outside the registers the index is kept in
//                            a cursor array in device memory.
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
  int32_t *last = (int32_t *)lds_raw, *anchor = last + n_sess;    // last chained event, its nominal end
  for (int s = lane; s < n_sess; s += WAVE) { last[s] = CH_NONE; anchor[s] = 0; }
  __syncthreads();
  for (int64_t base = lo; base < hi; base += WAVE) {
    const int cnt = hi - base < WAVE ? (int)(hi - base) : WAVE;
    const int32_t idx0 = (int32_t)(base - lo);
    int32_t t = 0, d = 0;
    uint32_t sk = 0;
    if (lane < cnt) { t = ev_time[base + lane]; d = ev_dur[base + lane]; sk = (uint32_t)ev_sk[base + lane]; }
    int32_t nx = -1, ny = -1;                   // this lane's record; ny = -1: in no chain
    for (int i = 0; i < cnt; i++) {             // in trace order: events of a tile may share a session
      const uint32_t ski = (uint32_t)lane_get((int)sk, i);
      const uint32_t kind = ski >> 24, s = ski & 0xFFFFFFu;
      const int32_t ti = lane_get(t, i), di = lane_get(d, i);
      const int32_t L = last[s];
      bool chained = false;
      if (kind == NBOS_EV_START) {
        chained = L == CH_NONE;
      } else if (L >= 0) {
        chained = true;
        const int32_t a = anchor[s];
        const int32_t th = ti > a ? ti - a : 0;
        if (L >= idx0) { if (lane == L - idx0) { nx = idx0 + i; ny = th; } }     // the predecessor is in this tile
        else if (lane == 0) chain[lo + L] = make_int2(idx0 + i, th);
      }
      wave_sync();
      if (chained) {
        if (lane == i) ny = 0;
        if (lane == 0) {
          last[s] = kind == NBOS_EV_END ? CH_CLOSED : idx0 + i;
          anchor[s] = kind == NBOS_EV_CELL ? ti + di : ti;
        }
      }
      wave_sync();
    }
    if (lane < cnt) chain[base + lane] = make_int2(nx, ny);
    __threadfence();                            // a later tile may overwrite one of these records
  }
}

template <uint32_t F>
__global__ void __launch_bounds__(WAVE) nbos_replay_closed_kernel(KParams p) {
  static_assert(Ctx<F>::closed, "instantiate with a closed-loop flag set");
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int rep = blockIdx.x;
  const int lane = threadIdx.x;
  if (rep >= p.n_replays) return;

  const int trace = p.trace_of_replay[rep];
  const int64_t ev_lo = p.ev_offset[trace], ev_hi = p.ev_offset[trace + 1];
  const int s_lo = p.sess_offset[trace];
  const int n_sess = p.sess_offset[trace + 1] - s_lo;

  const Lds m = lds_carve<true>(p, lds_raw);
  lds_init<true>(p, m, lane, s_lo, n_sess);

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
        // ---- S2: the earliest timer is due ----
        const int32_t now = r.q_head_t;
        const uint32_t key = (uint32_t)lane_get((int)c.qk, 0);
        const int32_t e = lane_get(c.qd, 0);
        int32_t x = lane_get(c.qx, 0), nx = lane_get(c.qnx, 0), nth = lane_get(c.qnth, 0);
        timer_pop(c, r);
        r.t_end = r.t_end > now ? r.t_end : now;
        const uint32_t s = key & 0xFFFFu, kind = key >> 16;
        wave_sync();
        const SessRec cur = m.sess[s];
        const uint32_t hw = uni((uint32_t)cur.x), fl = uni((uint32_t)cur.z);
        const int32_t tm = uni(cur.y);
        if (kind == QK_END) { end_session(c, r, s, hw, fl, now); continue; }
        if (!(x & CLX_LOADED)) {
          // scheduled straight into the registers: one round trip for the event's duration, kind and
          // chain record
          const int2 ch = c.cl_chain[e];
          x = uni(c.cl_dur[e]) | (int32_t)((uni((uint32_t)c.cl_sk[e]) >> 24) << 28) | CLX_LOADED;
          nx = uni(ch.x); nth = uni(ch.y);
        }
        r.cl_e = e; r.cl_x = x; r.cl_nx = nx; r.cl_nth = nth;
        const int32_t dur = x & 0x0FFFFFFF;
        if (kind == QK_RETRY) {
          attempt(c, r, s, hw, fl, now, tm, dur);
        } else if (((uint32_t)x >> 28 & 3u) == NBOS_EV_CELL) {        // the session submits its next cell (S4-S8)
          r.c_total++;
          const uint32_t st = fl & 7u;
          if (st == SS_PLACED && tm <= now && !(fl & SF_ENDING)) attempt(c, r, s, hw, fl & ~(SF_QONCE | (15u << 8)), now, now, dur);
          else if (st == SS_PLACED || st == SS_QUEUED) r.c_busy++;
          else r.c_unplaced++;
        } else {
          on_session_end(c, r, s, hw, tm, fl, now);     // S9
        }
        continue;
      }
      if (todo == 0) break;                 // draining and no timer is left
      todo &= todo - 1;
      const uint32_t s = (uint32_t)lane_get((int)vs, i) & 0xFFFFFFu;
      const uint32_t fl = uni((uint32_t)m.sess[s].z);
      r.t_end = r.t_end > t ? r.t_end : t;
      r.cl_e = (int32_t)(base - ev_lo) + i; r.cl_nx = lane_get(vnx, i); r.cl_nth = lane_get(vnth, i);
      session_start(c, r, s, fl, t);        // S3, S7; a placed session's first event is scheduled there
    }
    if (final) break;
  }
  write_stats(p, m, r, rep, lane);
}

}  // namespace ldsk
}  // namespace
