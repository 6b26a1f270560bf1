// nbos_kernel_lds.hpp — replay kernel with host state in LDS: any cluster size up to NBOS_MAX_HOSTS.
// Used when hosts_max > 64 (or on request). One workgroup per replay: one wave64 runs the replay; on
// clusters of 256 hosts or more, more waves of the workgroup (asleep at a barrier in between) take their
// share of every scan over all hosts (see "helper waves" below).
//
// LDS per replay
//   fin[h][8]    per-GPU "busy until" times, one 32-byte row per host. A GPU is committed at time t
//                iff fin > t; binding g GPUs for a cell (paper Section 3.3) = writing its finish time
//                into g free GPUs of the row. Completions need no timer: every timer due at or before
//                an item runs before that item and a completion only lowers C, so "released once
//                the clock has passed fin" is exact.
//   ready_at[h]  0 for initial hosts, NEVER while off, boot completion time while provisioning
//                (Section 3.4.2): readiness needs no timer either.
//   hsn[h]       subscribed GPUs S | replica count << 16 (Section 3.4.1).
//   mark[h]      scratch for the event-parallel rounds (lowest lane that chose the host), idle = ~0.
//   sess[s]      12 bytes: hosts word (3 x 10 bits + last executor slot), time word (busy-until, or
//                submit time while queued), flags.
//   due[s]       time of the session's timer while it waits outside the 64 sorted registers (NEVER: none
//                waits there); its kind is kept in the flags word, the duration of a queued cell in a
//                per-replay array in device memory.
//
// Serial path: one item (arrival, queued timer, auto-scaler period) per loop iteration; lane = host
// (strided) for every scan over hosts, ballot for feasibility, packed-key wave minimum for the choice
// (committed, subscribed, index: ties to the lowest host index). The election (Section 3.2.2) reads
// the 3 x 8 GPU words of the session's replica hosts with 24 lanes and counts with one ballot.
//
// Event-parallel rounds: lane = event. A run of consecutive cell arrivals of idle placed sessions
// with no timer due before them is evaluated at once: every lane gathers the rows of its session's
// three hosts, counts committed GPUs at its own time and elects. A lane's result equals the serial
// one if no earlier lane of the run binds GPUs on the host it chose (an earlier lane that binds on
// one of its other two hosts only makes that host a worse candidate: the choice stands) and no
// earlier lane failed its election (a failed election may migrate anywhere). The longest prefix
// with that property is committed at once - the chosen hosts are pairwise distinct by
// construction - and the rest is evaluated again. Counters are reduced over the prefix; the
// decision digest d*P + code is folded as d*P^n + sum(code_i * P^(n-1-i)) with a table of powers.
//
// Events: coalesced dword loads, one event per lane, next tile in flight while the current tile is
// consumed from registers. At tile start every lane prefetches its event's session record; cells of
// rejected / ended sessions and cells that arrive while their session's running cell outlasts them
// are counted in bulk and skipped.
#pragma once
#include "nbos_common.hpp"

namespace {
namespace ldsk {

constexpr int32_t MARK_FREE = 0x7FFFFFFF;

struct SessRec { int32_t x, y, z; };      // hosts word, time word, flags

struct Lds {
  unsigned long long *c64;
  uint32_t *c32, *hist;
  unsigned long long *ppow;    // P^0 .. P^64 of the digest multiplier
  int4 *fin;                   // two int4 per host
  int32_t *ready_at, *mark;
  int32_t *warm;               // [HP][4] when each pre-warmed container of a host is available (only with the pool)
  uint32_t *hsn;
  SessRec *sess;
  int32_t *due;                // [n_cap] time of a session's timer while it waits outside the registers, else NEVER
  int32_t *stage;              // [64] sessions whose timers move into the registers
  int32_t *mail;               // [MAIL_WORDS] what the helper waves are to do, and what they found (see helpers_go)
};

struct Regs {
  uint32_t n_dec, c_total, c_imm, c_started, c_busy, c_unplaced, reused, h0;
  int64_t sum_dur, g_exec;
  uint64_t digest;
  int32_t lazy_max, t_end;
  int32_t q_n, q_head_t;
  int32_t o_n, o_min_t;      // timers that wait in the session records: how many, a lower bound of the earliest
  uint32_t o_min_k;
  int32_t status;
  int32_t min_s;             // least subscription among hosts that are on, or -1 when stale
  uint64_t dirty;
  // closed loop: the event being handled, its duration and kind (packed as in Ctx::qx), its session's next
  // event and the think time before that; the time window the next refill takes
  int32_t cl_e, cl_x, cl_nx, cl_nth, cl_win;
};

template <uint32_t F>
struct Ctx {
  const KParams &p;
  Lds m;
  int lane;
  int32_t slim;              // floor(cap_milli * G * 3 / 1000): S + g <= slim is the cap test
  uint64_t *dlog;
  int32_t qt, qd;            // sorted timers, entry i in lane i
  uint32_t qk;
  uint32_t vsid;             // session id of this lane's event in the current tile (~0 if none)
  int32_t fu;                // lane g-1 (g = 1..8): no host can have g idle GPUs before this time
  // closed loop: sessions of the trace, the replay's cursors, the events of the trace; and with every
  // sorted timer what firing it needs: qd = the event's index, qx = its duration | kind << 28 |
  // CLX_LOADED (0: not loaded yet), qnx / qnth = its chain record
  int32_t n_sess;
  int32_t *cl_cur;
  const int32_t *cl_dur, *cl_sk;
  const int2 *cl_chain;
  int32_t qx, qnx, qnth;
  // lane g-1 (g = 1..8): no host that passes the subscription cap for a request of g GPUs can have g idle
  // GPUs before this time (0: nothing known). See cap_bound_* below.
  int32_t fc;
  int32_t *ovf_dur;          // open loop: [n_sess] durations of queued cells whose timer waits outside the registers
  int nw, wid;               // waves in the workgroup, this wave's number (0 runs the replay)
  bool dyn;                  // the dynamic limit can differ from the replay's cap (see dynamic_limit_matters)
  int32_t n_on;              // hosts that are on (ready or being provisioned): the wave's own copy of the counter
  static constexpr bool closed = closed_loop_instance(F);
  __device__ __forceinline__ uint32_t flags() const { return instance_flags<F>(p); }
};

// A session has at most one timer (the retry or deferred end of the cell under way; in a closed loop
// also its next event), so a timer that does not fit into the sorted registers waits in the session's
// own record: the kind in the flags word, the time in due[s] (NEVER: no timer waits there)
constexpr uint32_t CL_KIND_SHIFT = 13;
// Open loop: the duration word of a sorted RETRY timer (a duration is below 2^27) also says what is known
// about the retry. QD_LOOKED: the election of the queued cell has been worked out for the timer's time;
// QD_EFAIL: it fails there, whatever is bound until then (binding only takes idle GPUs away), and the
// retry is not the last one; bits 27-29 then hold the request g - 1. See retry_lookahead.
constexpr uint32_t QD_LOOKED = 1u << 31, QD_EFAIL = 1u << 30;
constexpr int QD_G_SHIFT = 27;
constexpr int32_t QD_DUR_MASK = (1 << QD_G_SHIFT) - 1;

template <uint32_t F>
__device__ __forceinline__ void sess_write(Ctx<F> &c, Regs &r, uint32_t s, uint32_t hw, int32_t tm, uint32_t fl) {
  if (c.lane == 0) { c.m.sess[s].x = (int)hw; c.m.sess[s].y = tm; c.m.sess[s].z = (int)fl; }
  r.dirty |= wballot(c.vsid == s);
}
template <uint32_t F>
__device__ __forceinline__ void sess_write_flag(Ctx<F> &c, Regs &r, uint32_t s, uint32_t fl) {
  if (c.lane == 0) c.m.sess[s].z = (int)fl;
  r.dirty |= wballot(c.vsid == s);
}

// ---- timers outside the sorted registers wait in the session records ---------------------------------
template <uint32_t F>
__device__ __forceinline__ void ovf_push(Ctx<F> &c, Regs &r, int32_t t, uint32_t k, int32_t d) {
  const uint32_t s = k & 0xFFFFu;
  if (c.lane == 0) {
    const uint32_t z = (uint32_t)c.m.sess[s].z;
    c.m.sess[s].z = (int)((z & ~(3u << CL_KIND_SHIFT)) | ((k >> 16) << CL_KIND_SHIFT));
    c.m.due[s] = t;
    if constexpr (!Ctx<F>::closed) {
      if ((k >> 16) == QK_RETRY) c.ovf_dur[s] = d & QD_DUR_MASK;
    }
  }
  if constexpr (!Ctx<F>::closed) r.dirty |= wballot(c.vsid == s);      // the flags word of the record has changed
  if (r.o_n == 0 || t < r.o_min_t || (t == r.o_min_t && k < r.o_min_k)) { r.o_min_t = t; r.o_min_k = k; }
  r.o_n++;
}

// Registers empty: all timers that are due within a window after the earliest one move
// from the session records into the registers at once, at most 64. A window takes whole instants, so
// everything taken is earlier than everything left behind whatever the kinds. The window adapts to
// the density of the timers (32 to 56 of the registers filled is the aim); if more than 64 timers wait
// for one and the same instant, the single earliest (time, kind, session) is taken. What firing the
// timers will need - the duration of a queued cell; in a closed loop their events' duration, kind and
// chain record - is gathered here, one lane per timer, in one or two round trips to device memory for
// the lot.
template <uint32_t F>
__device__ __forceinline__ void refill(Ctx<F> &c, Regs &r) {
  wave_sync();
  int cnt;
  int32_t left;                                  // earliest time left behind
  int32_t win = r.cl_win;
  for (;;) {
    const int64_t lim = (int64_t)r.o_min_t + win;
    const int32_t T = lim < NEVER - 1 ? (int32_t)lim : NEVER - 1;
    cnt = 0;
    int32_t mn = NEVER;                          // earliest time beyond the window, per lane
    // four sessions per lane and step (due[] is padded with NEVER to a multiple of four)
    const int4 *due4 = (const int4 *)c.m.due;
    for (int s0 = 4 * c.lane; s0 - 4 * c.lane < c.n_sess; s0 += 4 * WAVE) {
      const int4 d = s0 < c.n_sess ? due4[s0 >> 2] : make_int4(NEVER, NEVER, NEVER, NEVER);
      const int32_t lo = min(min(d.x, d.y), min(d.z, d.w));
      if (wballot(lo <= T) != 0) {               // rare: some of these timers are inside the window
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const int32_t dj = j == 0 ? d.x : j == 1 ? d.y : j == 2 ? d.z : d.w;
          const bool hit = dj <= T;
          const uint64_t b = wballot(hit);
          const int pos = cnt + lane_rank(b);
          if (hit && pos < WAVE) c.m.stage[pos] = s0 + j;
          cnt += __builtin_popcountll(b);
          mn = hit ? mn : (dj < mn ? dj : mn);
        }
      } else {
        mn = lo < mn ? lo : mn;
      }
    }
    left = (int32_t)wave_min((uint32_t)mn);
    if (cnt == 0) {                              // the stored bound was below the earliest time: use that
      if (left == NEVER) { r.o_n = 0; r.o_min_t = NEVER; return; }      // nothing waits (not reached: o_n counts them)
      r.o_min_t = left;
      continue;
    }
    if (cnt <= WAVE) break;
    if (win == 0) {
      // more than 64 timers at the instant o_min_t: the earliest by kind and session alone
      wave_sync();
      uint32_t best = 0xFFFFFFFFu;
      for (int s = c.lane; s < c.n_sess; s += WAVE) {
        if (c.m.due[s] == T) best = umin(best, ((((uint32_t)c.m.sess[s].z >> CL_KIND_SHIFT) & 3u) << 16) | (uint32_t)s);
      }
      best = wave_min(best);
      if (c.lane == 0) c.m.stage[0] = (int32_t)(best & 0xFFFFu);
      cnt = 1;
      left = T;
      break;
    }
    win = (int32_t)((int64_t)win * 40 / cnt);    // aim at 40 of the 64 registers
    wave_sync();
  }
  if (cnt < WAVE / 2 && win < CL_WIN_MAX) r.cl_win = win == 0 ? 1 : win + (win + 1) / 2;
  else if (cnt > 7 * WAVE / 8) r.cl_win = win - win / 4;
  else r.cl_win = win;
  wave_sync();
  // lane i < cnt takes the timer of session stage[i]
  const bool take = c.lane < cnt;
  uint32_t key = 0xFFFFFFFFu;
  int32_t t = NEVER, e = 0;
  if (take) {
    const int s = c.m.stage[c.lane];
    t = c.m.due[s];
    c.m.due[s] = NEVER;
    key = ((((uint32_t)c.m.sess[s].z >> CL_KIND_SHIFT) & 3u) << 16) | (uint32_t)s;
  }
  // the cursors / durations were written by lane 0 when the timers were scheduled: the fence makes this
  // wave's own stores visible to its other lanes
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  int32_t x = 0, nx = -1, nth = 0;
  if constexpr (Ctx<F>::closed) {
    if (take) e = c.cl_cur[key & 0xFFFFu];
    if (take && (key >> 16) != QK_END) {
      const int2 ch = c.cl_chain[e];
      x = c.cl_dur[e] | (int32_t)(((uint32_t)c.cl_sk[e] >> 24) << 28) | CLX_LOADED;
      nx = ch.x; nth = ch.y;
    }
  } else {
    if (take && (key >> 16) == QK_RETRY) e = c.ovf_dur[key & 0xFFFFu];       // qd carries the queued cell's duration
  }
  int rank = 0;
  for (int j = 0; j < cnt; j++) {
    const int32_t tj = lane_get(t, j);
    const uint32_t kj = (uint32_t)lane_get((int)key, j);
    rank += (tj < t || (tj == t && kj < key)) ? 1 : 0;
  }
  // lanes beyond cnt hold the largest key: their rank is cnt, any order among them will do
  const int dst = take ? rank : c.lane;
  c.qt = __builtin_amdgcn_ds_permute(dst << 2, t);
  c.qk = (uint32_t)__builtin_amdgcn_ds_permute(dst << 2, (int)key);
  c.qd = __builtin_amdgcn_ds_permute(dst << 2, e);
  if constexpr (Ctx<F>::closed) {
    c.qx = __builtin_amdgcn_ds_permute(dst << 2, x);
    c.qnx = __builtin_amdgcn_ds_permute(dst << 2, nx);
    c.qnth = __builtin_amdgcn_ds_permute(dst << 2, nth);
  }
  r.q_n = cnt;
  r.o_n -= cnt;
  r.o_min_t = r.o_n > 0 ? left : NEVER;
  r.o_min_k = 0;                                 // a lower bound: pushes for that very instant wait in the records
}

// ---- host helpers -------------------------------------------------------------------------------
// committed GPUs of host h at time `now` (GPUs beyond G keep fin = 0 and never count)
template <uint32_t F>
__device__ __forceinline__ int committed(const Ctx<F> &c, int h, int32_t now) {
  const int4 a = c.m.fin[2 * h], b = c.m.fin[2 * h + 1];
  return (a.x > now) + (a.y > now) + (a.z > now) + (a.w > now) + (b.x > now) + (b.y > now) + (b.z > now) + (b.w > now);
}

// bind g free GPUs of host h until `finish` (lanes 0..G-1 each look at one GPU)
template <uint32_t F>
__device__ __forceinline__ void bind_gpus(Ctx<F> &c, int h, int g, int32_t now, int32_t finish) {
  wave_sync();
  int32_t *row = (int32_t *)&c.m.fin[2 * h];
  const bool mine = c.lane < c.p.G;
  const int32_t f = mine ? row[c.lane] : NEVER;
  const bool fr = mine && f <= now;
  const int rank = lane_rank(wballot(fr));
  if (fr && rank < g) row[c.lane] = finish;
}

// ---- helper waves ------------------------------------------------------------------------------------
// A scan over all hosts is split by chunks of 64 hosts: wave w of the nw waves of the workgroup takes the
// chunks w, w + nw, ... The wave that runs the replay (wave 0) writes what is to be scanned into the mail
// words and meets the helpers at a barrier; each wave scans its chunks and reduces them; the helpers leave
// their results in the mail words, a second barrier, and wave 0 combines the nw results. Between scans the
// helpers sleep at the first barrier and take no issue slots. Every scan costs wave 0 exactly two barriers,
// every helper the same two; HC_EXIT ends the helpers' loop with one barrier on both sides.
// mail[0..3] = command, time, request g, room under the cap; mail[8 + 4 w + i] = result i of wave w.
enum { HC_EXIT = 0, HC_BEST_HOST, HC_EARLIEST_IDLE, HC_PLACE, HC_TICK };
// (more than four waves gain nothing measurable: 12 chunks of hosts on 4 / 6 / 8 / 12 waves take 269 / 265 / 266 /
// 269 ms on the 768-host workload, and a workgroup of more than 256 threads leaves the compiler fewer registers)
constexpr int MAX_WAVES = 4, MAIL_WORDS = 8 + 4 * MAX_WAVES;

template <uint32_t F>
__device__ __forceinline__ void helpers_go(const Ctx<F> &c, int cmd, int32_t now, int g, int32_t room) {
  if (c.nw == 1) return;
  if (c.lane == 0) *(int4 *)c.m.mail = make_int4(cmd, now, g, room);
  __syncthreads();
}
template <uint32_t F>
__device__ __forceinline__ void helpers_done(const Ctx<F> &c) {
  if (c.nw > 1) __syncthreads();
}
// result i of helper wave w, as a uniform value (after helpers_done)
template <uint32_t F>
__device__ __forceinline__ uint32_t helper_result(const Ctx<F> &c, int w, int i) {
  return uni((uint32_t)c.m.mail[8 + 4 * w + i]);
}

// lowest host index that is off (the caller has checked that one exists)
template <uint32_t F>
__device__ __forceinline__ int find_off_host(const Ctx<F> &c) {
  wave_sync();
  for (int base = 0; base < c.p.HP; base += WAVE) {
    const int h = base + c.lane;
    const uint64_t off = wballot(h < c.p.Hmax && c.m.ready_at[h] == NEVER);
    if (off) return base + (int)__builtin_ctzll(off);
  }
  return 0;
}

template <uint32_t F>
__device__ __forceinline__ int boot_host(Ctx<F> &c, Regs &r, int32_t now, uint32_t hs_new) {
  const int h = find_off_host(c);
  const int32_t ra = now + c.p.boot;
  if (c.lane == 0) { c.m.ready_at[h] = ra; c.m.hsn[h] = hs_new; }
  if (c.flags() & NBOS_F_WARM_POOL) {         // its pre-warmed containers are there once it is up
    if (c.lane < 4) c.m.warm[4 * h + c.lane] = ra + c.p.prewarm;
  }
  c.fu = c.fu < ra ? c.fu : ra;               // a new host may have idle GPUs from then on
  c.fc = c.fc < ra ? c.fc : ra;
  r.min_s = -1;
  c32_add(c.m, c.lane, CS_NON, 1u);
  c.n_on++;
  c64_add(c.m, c.lane, CL_PROV, -(int64_t)c.p.G * now);
  c32_add(c.m, c.lane, CS_SO, 1u);
  r.lazy_max = r.lazy_max > ra ? r.lazy_max : ra;
  return h;
}

// Best host for one more replica with request g that is to bind its GPUs at once: ready, under the cap
// (S <= room), with g idle GPUs now; smallest (committed, subscribed, index). Returns the packed key
// (host in the low 10 bits) or 0xFFFFFFFF. any_idle: some ready host has g idle GPUs, cap aside.
// _part: this wave's chunks of hosts.
template <uint32_t F>
__device__ __forceinline__ uint32_t best_host_part(const Ctx<F> &c, int32_t now, int g, int32_t room, bool &any_idle) {
  uint32_t best = 0xFFFFFFFFu;
  bool idle_seen = false;
  for (int h = c.wid * WAVE + c.lane; h < c.p.HP; h += WAVE * c.nw) {
    const int32_t ra = c.m.ready_at[h];
    const int S = (int)(c.m.hsn[h] & 0xFFFFu);
    const bool capped = ra <= now && S <= room;
    // the GPU rows are only read for a chunk of hosts in which somebody passes the cap (or while it
    // is still open whether any host has g idle GPUs)
    if (wballot(capped) == 0 && idle_seen) continue;
    const int C = committed(c, h, now);
    const bool roomy = ra <= now && C + g <= c.p.G;
    idle_seen = idle_seen || wballot(roomy) != 0;
    const uint32_t key = ((uint32_t)C << 22) | ((uint32_t)S << 10) | (uint32_t)h;
    if (capped && roomy) best = umin(best, key);
  }
  any_idle = idle_seen;
  return wave_min(best);
}

template <uint32_t F>
__device__ __forceinline__ uint32_t best_host(const Ctx<F> &c, int32_t now, int g, int32_t room, bool &any_idle) {
  wave_sync();
  helpers_go(c, HC_BEST_HOST, now, g, room);
  uint32_t key = best_host_part(c, now, g, room, any_idle);
  helpers_done(c);
  for (int w = 1; w < c.nw; w++) {
    key = umin(key, helper_result(c, w, 0));
    any_idle = any_idle || helper_result(c, w, 1) != 0;
  }
  return key;
}

// least subscribed-GPU count among the hosts that are on (ready or being provisioned)
template <uint32_t F>
__device__ __forceinline__ int32_t min_subscription(const Ctx<F> &c) {
  wave_sync();
  uint32_t best = 0xFFFFu;
  for (int h = c.lane; h < c.p.HP; h += WAVE) {
    const uint32_t S = c.m.hsn[h] & 0xFFFFu;
    if (c.m.ready_at[h] != NEVER) best = umin(best, S);
  }
  return (int32_t)wave_min(best);
}

__device__ __forceinline__ void order2(int32_t &a, int32_t &b) {
  const int32_t lo = a < b ? a : b, hi = a < b ? b : a;
  a = lo; b = hi;
}

// the busy-until times of one host's GPUs in ascending order (GPUs beyond G count as never free):
// the 19-comparator network for 8 inputs; returns the g-th smallest
__device__ __forceinline__ int32_t kth_free_time(const int4 a, const int4 b, int G, int g) {
  int32_t v0 = a.x, v1 = G > 1 ? a.y : NEVER, v2 = G > 2 ? a.z : NEVER, v3 = G > 3 ? a.w : NEVER;
  int32_t v4 = G > 4 ? b.x : NEVER, v5 = G > 5 ? b.y : NEVER, v6 = G > 6 ? b.z : NEVER, v7 = G > 7 ? b.w : NEVER;
  order2(v0, v1); order2(v2, v3); order2(v4, v5); order2(v6, v7);
  order2(v0, v2); order2(v1, v3); order2(v4, v6); order2(v5, v7);
  order2(v1, v2); order2(v5, v6);
  order2(v0, v4); order2(v1, v5); order2(v2, v6); order2(v3, v7);
  order2(v2, v4); order2(v3, v5);
  order2(v1, v2); order2(v3, v4); order2(v5, v6);
  return g == 1 ? v0 : g == 2 ? v1 : g == 3 ? v2 : g == 4 ? v3 : g == 5 ? v4 : g == 6 ? v5 : g == 7 ? v6 : v7;
}

// Earliest time at which some host that is on could have g idle GPUs if nothing new were committed:
// min over hosts of max(ready_at, g-th smallest busy-until time of the host's GPUs). Later commits
// only push it back, so no election or migration for a request of g GPUs can succeed before it, as
// long as no host is added (boot_host lowers the stored bound). `capped`: the same minimum over the
// hosts that hold at most `room` subscribed GPUs, i.e. that pass the subscription cap for the request
// (Section 3.4.1): no migration target before it, as long as no host is added and no host's
// subscription shrinks (cap_bound_host_freed lowers the stored bound then). One lane sorts one host's row.
template <uint32_t F>
__device__ __forceinline__ int32_t earliest_idle_part(const Ctx<F> &c, int g, int32_t room, int32_t &capped) {
  const int G = c.p.G;
  int32_t best = NEVER, best_cap = NEVER;
  for (int h = c.wid * WAVE + c.lane; h < c.p.HP; h += WAVE * c.nw) {
    int32_t y = kth_free_time(c.m.fin[2 * h], c.m.fin[2 * h + 1], G, g);
    const int32_t ra = c.m.ready_at[h];
    y = y > ra ? y : ra;
    best = best < y ? best : y;
    const int32_t yc = (int32_t)(c.m.hsn[h] & 0xFFFFu) <= room ? y : NEVER;
    best_cap = best_cap < yc ? best_cap : yc;
  }
  capped = (int32_t)wave_min((uint32_t)best_cap);
  return (int32_t)wave_min((uint32_t)best);
}

template <uint32_t F>
__device__ __forceinline__ int32_t earliest_idle(const Ctx<F> &c, int g, int32_t room, int32_t &capped) {
  wave_sync();
  helpers_go(c, HC_EARLIEST_IDLE, 0, g, room);
  int32_t best = earliest_idle_part(c, g, room, capped);
  helpers_done(c);
  for (int w = 1; w < c.nw; w++) {
    const int32_t b = (int32_t)helper_result(c, w, 0), bc = (int32_t)helper_result(c, w, 1);
    best = best < b ? best : b;
    capped = capped < bc ? capped : bc;
  }
  return best;
}

// Host h now holds s_new subscribed GPUs, fewer than before (a session ended, a replica moved away): it
// may newly pass the cap for requests of up to slim - s_new GPUs, so the stored bounds of those requests
// drop to the time at which this host could have the GPUs idle. Lane g-1 works out the bound for g.
template <uint32_t F>
__device__ __forceinline__ void cap_bound_host_freed(Ctx<F> &c, int h, int32_t s_new, int32_t now) {
  if ((c.flags() & NBOS_F_DYNAMIC_SR) && c.dyn) return;   // the limit moves with the cluster's sums: no bound is kept
  if (wballot(c.lane < NGPU && c.fc > now) == 0) return;  // every bound lies in the past already: as good as none
  wave_sync();
  const int g = (c.lane & 7) + 1;
  int32_t y = kth_free_time(c.m.fin[2 * h], c.m.fin[2 * h + 1], c.p.G, g);
  const int32_t ra = c.m.ready_at[h];
  y = y > ra ? y : ra;
  if (c.lane < NGPU && s_new + g <= c.slim && y < c.fc) c.fc = y;
}

// ---- closed loop: the session's next event is due one think time after `base` --------------------
// r.cl_nx / r.cl_nth: the event after the one being handled and the think time before it. The timer
// carries the event's index; the cursor keeps it for the time the timer waits outside the registers.
template <uint32_t F>
__device__ __forceinline__ void cl_schedule(Ctx<F> &c, Regs &r, uint32_t s, int32_t base) {
  const int32_t e = r.cl_nx;
  if (e < 0) return;
  const int64_t t = (int64_t)base + r.cl_nth;
  if (t >= 0x7FFFFFFFLL) { r.status = NBOS_E_RANGE; return; }
  if (c.lane == 0) c.cl_cur[s] = e;
  timer_push(c, r, (int32_t)t, QK_NEXT, s, e);
}

// Placement candidates among this wave's chunks of hosts (Sections 3.2.1, 3.4.1): ready and under the cap;
// one pass computes every host's key (strided over the lanes), three minima pick the three best
// (0xFFFFFFFF where there are fewer). MAXCH: the most chunks of 64 hosts a wave can have (all 16 for a wave
// on its own, 4 with MAX_WAVES waves).
template <int MAXCH, uint32_t F>
__device__ __forceinline__ void place_part(const Ctx<F> &c, int32_t now, int32_t room, uint32_t &m0, uint32_t &m1,
                                           uint32_t &m2) {
  uint32_t keys[MAXCH];
#pragma unroll
  for (int j = 0; j < MAXCH; j++) {
    keys[j] = 0xFFFFFFFFu;
    const int h = (j * c.nw + c.wid) * WAVE + c.lane;
    if (h - c.lane < c.p.HP) {
      const int S = (int)(c.m.hsn[h] & 0xFFFFu);
      if (c.m.ready_at[h] <= now && S <= room)
        keys[j] = ((uint32_t)committed(c, h, now) << 22) | ((uint32_t)S << 10) | (uint32_t)h;
    }
  }
  uint32_t out[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
#pragma unroll
  for (int round = 0; round < 3; round++) {
    uint32_t best = 0xFFFFFFFFu;
#pragma unroll
    for (int j = 0; j < MAXCH; j++) best = umin(best, keys[j]);
    const uint32_t m = wave_min(best);
    if (m == 0xFFFFFFFFu) break;
    out[round] = m;
#pragma unroll
    for (int j = 0; j < MAXCH; j++) keys[j] = keys[j] == m ? 0xFFFFFFFFu : keys[j];
  }
  m0 = out[0]; m1 = out[1]; m2 = out[2];
}

// ---- SESSION_START: Sections 3.2.1, 3.4.1, 3.4.2 -----------------------------------------------
template <uint32_t F>
__device__ __forceinline__ void session_start(Ctx<F> &c, Regs &r, uint32_t s, uint32_t fl, int32_t now) {
  if ((fl & 7u) != SS_UNPLACED) return;
  const int g = (int)((fl >> 3) & 7u) + 1;
  const int32_t room = cap_room(c, g);
  wave_sync();
  helpers_go(c, HC_PLACE, now, g, room);
  uint32_t m0, m1, m2;
  if (c.nw == MAX_WAVES) place_part<NBOS_MAX_HOSTS / WAVE / MAX_WAVES>(c, now, room, m0, m1, m2);
  else place_part<NBOS_MAX_HOSTS / WAVE>(c, now, room, m0, m1, m2);
  if (c.nw > 1) {
    // the three best of every wave meet in the mail words: the three best of those are the hosts
    if (c.lane == 0) { c.m.mail[8] = (int)m0; c.m.mail[9] = (int)m1; c.m.mail[10] = (int)m2; }
    helpers_done(c);
    uint32_t key = 0xFFFFFFFFu;
    if (c.lane < 4 * c.nw && (c.lane & 3) != 3) key = (uint32_t)c.m.mail[8 + c.lane];
    m0 = wave_min(key);
    key = key == m0 ? 0xFFFFFFFFu : key;
    m1 = wave_min(key);
    key = key == m1 ? 0xFFFFFFFFu : key;
    m2 = wave_min(key);
  }
  int pick0 = -1, pick1 = -1, pick2 = -1, k = 0;
  if (m0 != 0xFFFFFFFFu) { pick0 = (int)(m0 & 1023u); k = 1; }
  if (m1 != 0xFFFFFFFFu) { pick1 = (int)(m1 & 1023u); k = 2; }
  if (m2 != 0xFFFFFFFFu) { pick2 = (int)(m2 & 1023u); k = 3; }
  const int missing = 3 - k;
  if (missing > 0) {
    const int n_on = c.n_on;
    if (!((c.flags() & NBOS_F_SCALE_OUT) && n_on + missing <= c.p.Hmax)) {
      sess_write_flag(c, r, s, (fl & ~7u) | SS_REJECTED);
      c32_add(c.m, c.lane, CS_REJECTED, 1u);
      decide(c, r, now, NBOS_D_REJECT, s, 0, 0);
      return;
    }
  }
  const uint32_t add = (uint32_t)g | (1u << 16);
  uint32_t hw = 0;
#pragma unroll
  for (int i = 0; i < 3; i++) {
    int h = i == 0 ? pick0 : (i == 1 ? pick1 : pick2);
    if (i < k) {
      r.min_s = -1;
      if (c.lane == 0) atomicAdd(&c.m.hsn[h], add);          // (one ds_add, nothing to wait for)
      decide(c, r, now, NBOS_D_PLACE, s, (uint32_t)i, (uint32_t)h);
    } else {
      h = boot_host(c, r, now, add);
      decide(c, r, now, NBOS_D_PLACE_NEW, s, (uint32_t)i, (uint32_t)h);
    }
    hw |= (uint32_t)h << (10 * i);
  }
  if (missing > 0) c32_max(c.m, c.lane, CS_PEAK, (uint32_t)c.n_on);
  sess_write(c, r, s, hw, 0, (fl & ~7u) | SS_PLACED);
  c32_add(c.m, c.lane, CS_PLACED, 1u);
  c32_add(c.m, c.lane, CS_SUMS, (uint32_t)(3 * g));
  c32_add(c.m, c.lane, CS_OPENG, (uint32_t)g);
  c64_add(c.m, c.lane, CL_SUB, -(int64_t)(3 * g) * now);
  c64_add(c.m, c.lane, CL_RESV, -(int64_t)g * now);
  c32_add(c.m, c.lane, CS_NREP, 3u);
  c64_add(c.m, c.lane, CL_REPL, -(int64_t)3 * now);
  if constexpr (Ctx<F>::closed) cl_schedule(c, r, s, now);
}

// the replicas of session s give their subscriptions back at time `now`
template <uint32_t F>
__device__ __forceinline__ void end_session(Ctx<F> &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int32_t now) {
  const int g = (int)((fl >> 3) & 7u) + 1;
  const uint32_t sub = (uint32_t)g | (1u << 16);
  if (c.lane < 3) {
    const int h = (int)((hw >> (10 * c.lane)) & 1023u);
    atomicSub(&c.m.hsn[h], sub);                // three distinct hosts, one lane each
  }
  r.min_s = -1;
  if (!((c.flags() & NBOS_F_DYNAMIC_SR) && c.dyn)) {
    wave_sync();
#pragma unroll
    for (int i = 0; i < 3; i++) {
      const int h = (int)((hw >> (10 * i)) & 1023u);
      cap_bound_host_freed(c, h, (int32_t)(uni(c.m.hsn[h]) & 0xFFFFu), now);
    }
  }
  sess_write_flag(c, r, s, (fl & ~(7u | SF_ENDING)) | SS_ENDED);
  c32_add(c.m, c.lane, CS_SUMS, (uint32_t)(-3 * g));
  c64_add(c.m, c.lane, CL_SUB, (int64_t)(3 * g) * now);
  c32_add(c.m, c.lane, CS_NREP, (uint32_t)-3);
  c64_add(c.m, c.lane, CL_REPL, (int64_t)3 * now);
}

// ---- a cell starts on (slot, host): Section 3.3 and the metrics of sections "Resource Usage & Efficiency", "Interactivity" and "Task Completion Time" ---------
template <uint32_t F>
__device__ __forceinline__ void start_cell(Ctx<F> &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int slot, int host,
                                           int32_t now, int32_t start, int32_t t_submit, int32_t dur,
                                           uint32_t outcome) {
  const int g = (int)((fl >> 3) & 7u) + 1;
  if constexpr (Ctx<F>::closed) {             // the lag of a closed loop is not bounded in advance
    if ((int64_t)start + dur >= 0x7FFFFFFFLL) { r.status = NBOS_E_RANGE; return; }
  }
  const int32_t finish = start + dur;
  const int32_t delay = start - t_submit;
  r.c_started++;
  r.sum_dur += dur;
  r.g_exec += (int64_t)g * dur;
  const uint32_t last = hw >> 30;               // 0 none, else slot + 1
  if (last == (uint32_t)slot + 1u) r.reused++;
  hw = (hw & 0x3FFFFFFFu) | ((uint32_t)(slot + 1) << 30);
  hw = (hw & ~(1023u << (10 * slot))) | ((uint32_t)host << (10 * slot));
  const uint32_t nfl = (fl & ~(7u | SF_QONCE | (15u << 8))) | SS_PLACED;
  if (delay == 0) {
    r.h0++;                                     // histogram bin 0 lives in a register
    if (c.lane == 0) {
      c.m.sess[s].x = (int)hw; c.m.sess[s].y = finish;
      if (nfl != fl) c.m.sess[s].z = (int)nfl;
    }
  } else {
    int b = 32 - __builtin_clz((uint32_t)delay);
    b = b > 31 ? 31 : b;
    if (c.lane == 0) {
      c.m.sess[s].x = (int)hw; c.m.sess[s].y = finish; c.m.sess[s].z = (int)nfl;
      atomicAdd(&c.m.hist[b], 1u);
      atomicAdd(&c.m.c64[CL_SUMDELAY], (unsigned long long)delay);
      atomicMax(&c.m.c32[CS_MAXDELAY], (uint32_t)delay);
      atomicAdd(&c.m.c64[CL_GWAIT], (unsigned long long)((int64_t)g * (start - now)));
    }
  }
  r.dirty |= wballot(c.vsid == s);
  r.lazy_max = r.lazy_max > finish ? r.lazy_max : finish;
  decide(c, r, now, outcome, s, (uint32_t)slot, (uint32_t)host);
  if (fl & SF_ENDING) timer_push(c, r, finish, QK_END, s, 0);
  if constexpr (Ctx<F>::closed) cl_schedule(c, r, s, finish);
}

// ---- one attempt to run the pending cell of session s at time `now` -----------------------------
// Returns what the attempt did to the things retry_horizon looks at: NEVER = nothing (the cell started by
// election: GPUs were bound, no timer pushed); a time = a retry timer for that time was pushed and nothing
// else changed; -1 = anything else (subscriptions moved, a host was added, bounds were lowered).
template <uint32_t F>
__device__ __forceinline__ int32_t attempt(Ctx<F> &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int32_t now,
                                           int32_t t_submit, int32_t dur) {
  PROF_SUB_BEGIN();
  wave_sync();
  const int G = c.p.G;
  const int g = (int)((fl >> 3) & 7u) + 1;
  const uint32_t h0 = hw & 1023u, h1 = (hw >> 10) & 1023u, h2 = (hw >> 20) & 1023u;
  // Known in advance that no host has g idle GPUs yet? Then neither election nor migration can work.
  const bool hopeless = now < lane_get(c.fu, g - 1);
  // (a) election, Section 3.2.2: lanes 0..23 = (replica, GPU) of the session's hosts
  int rr = c.lane >> 3;
  rr = rr > 2 ? 2 : rr;
  const int k = c.lane & 7;
  const int hr = (int)((hw >> (10 * rr)) & 1023u);
  const bool act = c.lane < 24;
  int32_t *row = (int32_t *)&c.m.fin[2 * hr];
  const int32_t f = row[k];
  const int32_t ra = c.m.ready_at[hr];
  const uint64_t busy = wballot(act && f > now);
  const uint64_t rdy = wballot(ra <= now);
  const int C0 = __builtin_popcount((uint32_t)busy & 0xFFu), C1 = __builtin_popcount((uint32_t)(busy >> 8) & 0xFFu),
            C2 = __builtin_popcount((uint32_t)(busy >> 16) & 0xFFu);
  const int ok0 = (int)(rdy & 1u), ok1 = (int)((rdy >> 8) & 1u), ok2 = (int)((rdy >> 16) & 1u);
  if (!hopeless) {
    const uint32_t k0 = (ok0 && C0 + g <= G) ? (((uint32_t)C0 << 12) | (h0 << 2) | 0u) : 0xFFFFFFFFu;
    const uint32_t k1 = (ok1 && C1 + g <= G) ? (((uint32_t)C1 << 12) | (h1 << 2) | 1u) : 0xFFFFFFFFu;
    const uint32_t k2 = (ok2 && C2 + g <= G) ? (((uint32_t)C2 << 12) | (h2 << 2) | 2u) : 0xFFFFFFFFu;
    uint32_t kb = umin(k0, umin(k1, k2));
    if (c.flags() & NBOS_F_STICKY_EXECUTOR) {
      // variant: the replica that ran the previous cell leads again if its host can bind
      const uint32_t last = hw >> 30;
      const uint32_t kp = last == 1u ? k0 : (last == 2u ? k1 : (last == 3u ? k2 : 0xFFFFFFFFu));
      if (kp != 0xFFFFFFFFu) kb = kp;
    }
    if (kb != 0xFFFFFFFFu) {
      const int lead = (int)(kb & 3u), hl = (int)((kb >> 2) & 1023u);
      const bool fr = act && (c.lane >> 3) == lead && k < G && f <= now;
      const int rank = lane_rank(wballot(fr));
      if (fr && rank < g) row[k] = now + dur;
      if (now == t_submit) r.c_imm++;
      start_cell(c, r, s, hw, fl, lead, hl, now, now, t_submit, dur, NBOS_D_START);
      return (Ctx<F>::closed || (fl & SF_ENDING)) ? -1 : NEVER;      // (those push a timer of their own)
    }
  }
  PROF_SUB(PC_A_ELECT);
  // (b), (c): a target exists? Only then is the replica to move worked out.
  uint32_t tkey = 0xFFFFFFFFu;
  if (!hopeless && (c.flags() & NBOS_F_MIGRATE)) {
    if ((c.flags() & NBOS_F_DYNAMIC_SR) && c.dyn) {
      // the cap alone may rule every host out: S_h + g <= limit fails even for the least subscribed
      if (r.min_s < 0) r.min_s = min_subscription(c);
      const int32_t room = cap_room(c, g);
      if (r.min_s <= room) {
        bool any_idle;
        tkey = best_host(c, now, g, room, any_idle);
        if (!any_idle) {
          // No host at all with g idle GPUs: work out when the first one could have them, once, for
          // every later attempt with a request of g or more.
          int32_t unused;
          const int32_t bound = earliest_idle(c, g, room, unused);
          if (c.lane >= g - 1 && c.fu < bound) c.fu = bound;
        }
      }
    } else if (now >= lane_get(c.fc, g - 1)) {
      // (before that time no host that passes the cap can have the GPUs idle: nothing to look for)
      const int32_t room = c.slim - g;
      bool any_idle;
      tkey = best_host(c, now, g, room, any_idle);
      if (tkey == 0xFFFFFFFFu) {
        // No target: work out when the first host could have g idle GPUs, and the first one among those
        // under the cap, once, for every later attempt with a request of g or more.
        int32_t under_cap;
        const int32_t bound = earliest_idle(c, g, room, under_cap);
        if (c.lane >= g - 1) {
          if (c.fu < bound) c.fu = bound;
          if (c.fc < under_cap) c.fc = under_cap;
        }
      }
    }
  }
  PROF_SUB(PC_A_TARGET);
  bool grow = false;
  if (tkey == 0xFFFFFFFFu && (c.flags() & NBOS_F_SCALE_OUT)) grow = c.n_on < c.p.Hmax;
  if (tkey != 0xFFFFFFFFu || grow) {
    // the replica on the fullest ready host moves (ties: lowest host); booting ones only if all are
    const int any_ready = ok0 | ok1 | ok2;
    const uint32_t v0 = (!any_ready || ok0) ? (((uint32_t)(8 - C0) << 12) | (h0 << 2) | 0u) : 0xFFFFFFFFu;
    const uint32_t v1 = (!any_ready || ok1) ? (((uint32_t)(8 - C1) << 12) | (h1 << 2) | 1u) : 0xFFFFFFFFu;
    const uint32_t v2 = (!any_ready || ok2) ? (((uint32_t)(8 - C2) << 12) | (h2 << 2) | 2u) : 0xFFFFFFFFu;
    const uint32_t vb = umin(v0, umin(v1, v2));
    const int victim = (int)(vb & 3u), hv = (int)((vb >> 2) & 1023u);
    const uint32_t moved = (uint32_t)g | (1u << 16);
    if (tkey != 0xFFFFFFFFu) {
      // (b) migration, Section 3.2.3: the target binds the GPUs at once. A ready host of this session
      // with g idle GPUs would have won the election, so none of its hosts can show up as a target.
      const int dst = (int)(tkey & 1023u);
      int32_t start = now + c.p.migr;
      uint32_t outcome = NBOS_D_MIGRATE;
      if (c.flags() & NBOS_F_WARM_POOL) {
        // Section 3.2.3: the target's pre-warmed container that has been available longest, if any
        // is available now, shortens the start; its replacement is there one pre-warm time later
        wave_sync();
        const uint32_t av = c.lane < c.p.warm_n ? (uint32_t)c.m.warm[4 * dst + c.lane] : 0xFFFFFFFFu;
        const uint32_t first = wave_min(av);
        if ((int32_t)first <= now) {
          const int w = (int)__builtin_ctzll(wballot(av == first));
          if (c.lane == w) c.m.warm[4 * dst + w] = now + c.p.prewarm;
          start = now + c.p.warm_migr;
          outcome = NBOS_D_MIGRATE_WARM;
          c32_add(c.m, c.lane, CS_MIGRWARM, 1u);
        }
      }
      if (c.lane == 0) { atomicSub(&c.m.hsn[hv], moved); atomicAdd(&c.m.hsn[dst], moved); }
      r.min_s = -1;
      wave_sync();
      cap_bound_host_freed(c, hv, (int32_t)(uni(c.m.hsn[hv]) & 0xFFFFu), now);
      PROF_SUB(PC_A_VICTIM);
      bind_gpus(c, dst, g, now, start + dur);
      c32_add(c.m, c.lane, CS_MIGR, 1u);
      start_cell(c, r, s, hw, fl, victim, dst, now, start, t_submit, dur, outcome);
      PROF_SUB(PC_A_BIND);
    } else {
      // (c) a new host for the cell, Section 3.4.2: reserved and bound before it is up
      const int32_t start = now + c.p.boot + c.p.migr;
      if (c.lane == 0) atomicSub(&c.m.hsn[hv], moved);
      r.min_s = -1;
      wave_sync();
      cap_bound_host_freed(c, hv, (int32_t)(uni(c.m.hsn[hv]) & 0xFFFFu), now);
      const int h = boot_host(c, r, now, moved);
      c32_max(c.m, c.lane, CS_PEAK, (uint32_t)c.n_on);
      bind_gpus(c, h, g, now, start + dur);
      c32_add(c.m, c.lane, CS_MIGR, 1u);
      start_cell(c, r, s, hw, fl, victim, h, now, start, t_submit, dur, NBOS_D_SCALE_CELL);
    }
    return -1;
  }
  // (d) queue and retry periodically, then give up, Section 3.2.3
  int retries = (int)((fl >> 8) & 15u);
  if (retries < c.p.max_retries) {
    retries++;
    const uint32_t nfl = (fl & ~(7u | (15u << 8))) | SS_QUEUED | SF_QONCE | ((uint32_t)retries << 8);
    if (!(fl & SF_QONCE)) {                      // first time in the queue: the submit time goes in
      c32_add(c.m, c.lane, CS_QUEUED, 1u);
      if (c.lane == 0) { c.m.sess[s].y = t_submit; c.m.sess[s].z = (int)nfl; }
    } else {
      if (c.lane == 0) c.m.sess[s].z = (int)nfl;
    }
    r.dirty |= wballot(c.vsid == s);
    if constexpr (Ctx<F>::closed) {
      if ((int64_t)t_submit + (int64_t)retries * c.p.retry_iv >= 0x7FFFFFFFLL) { r.status = NBOS_E_RANGE; return -1; }
    }
    // closed loop: every timer carries its event (the cursor still points at the cell under way)
    if constexpr (Ctx<F>::closed) timer_push(c, r, t_submit + retries * c.p.retry_iv, QK_RETRY, s, r.cl_e, r.cl_x, r.cl_nx, r.cl_nth);
    else timer_push(c, r, t_submit + retries * c.p.retry_iv, QK_RETRY, s, dur);
    return t_submit + retries * c.p.retry_iv;
  }
  c32_add(c.m, c.lane, CS_ABORTED, 1u);
  decide(c, r, now, NBOS_D_ABORT, s, 0, 0);
  const uint32_t nfl = (fl & ~(7u | SF_QONCE | (15u << 8))) | SS_PLACED;
  sess_write(c, r, s, hw, 0, nfl);
  if (fl & SF_ENDING) end_session(c, r, s, hw, nfl, now);
  if constexpr (Ctx<F>::closed) cl_schedule(c, r, s, now);
  return -1;
}

// Sum of a per-lane value below 2^26 over the wave as a 64-bit uniform value: exact 32-bit sums per
// row of 16 lanes (DPP butterfly), the four rows added on the scalar unit.
__device__ __forceinline__ uint64_t wave_sum(uint32_t v) {
  v += dpp<0xB1>(v);
  v += dpp<0x4E>(v);
  v += dpp<0x141>(v);
  v += dpp<0x140>(v);
  return (uint64_t)(uint32_t)lane_get((int)v, 0) + (uint64_t)(uint32_t)lane_get((int)v, 16) +
         (uint64_t)(uint32_t)lane_get((int)v, 32) + (uint64_t)(uint32_t)lane_get((int)v, 48);
}

// ---- auto-scaler period (Section 3.4.2) -----------------------------------------------------------
// release the highest-numbered ready host without replicas (the caller has checked that one exists)
template <uint32_t F>
__device__ __forceinline__ void release_host(Ctx<F> &c, Regs &r, int32_t now) {
  int victim = -1;
  wave_sync();
  for (int base = c.p.HP - WAVE; base >= 0 && victim < 0; base -= WAVE) {
    const int h = base + c.lane;
    const uint64_t e = wballot(c.m.ready_at[h] <= now && (c.m.hsn[h] >> 16) == 0);
    if (e) victim = base + 63 - (int)__builtin_clzll(e);
  }
  if (c.lane == 0) c.m.ready_at[victim] = NEVER;
  r.min_s = -1;
  c32_add(c.m, c.lane, CS_NON, (uint32_t)-1);
  c.n_on--;
  c64_add(c.m, c.lane, CL_PROV, (int64_t)c.p.G * now);
  c32_add(c.m, c.lane, CS_SI, 1u);
  decide(c, r, now, NBOS_D_SCALE_IN, 0, 0, (uint32_t)victim);
}

// this wave's chunks of hosts: ready hosts, ready hosts without replicas, committed GPUs (auto-scaler only)
template <uint32_t F>
__device__ __forceinline__ void tick_part(const Ctx<F> &c, int32_t now, int &A, int &Z, uint32_t &sum_c) {
  const bool autoscale = (c.flags() & NBOS_F_AUTOSCALE) != 0;
  A = 0; Z = 0;
  uint32_t busy = 0;                       // this lane's share of sum C
  for (int h = c.wid * WAVE + c.lane; h < c.p.HP; h += WAVE * c.nw) {
    const bool ready = c.m.ready_at[h] <= now;
    A += __builtin_popcountll(wballot(ready));
    Z += __builtin_popcountll(wballot(ready && (c.m.hsn[h] >> 16) == 0));
    if (autoscale) busy += (uint32_t)committed(c, h, now);
  }
  sum_c = autoscale ? (uint32_t)wave_sum(busy) : 0u;
}

// What the helper waves (wave 1 and up) do for the whole kernel: see "helper waves" above.
template <uint32_t F>
__device__ __forceinline__ void helper_loop(const Ctx<F> &c) {
  for (;;) {
    __syncthreads();
    const int4 cmd = *(const int4 *)c.m.mail;
    const int what = uni(cmd.x), g = uni(cmd.z);
    const int32_t now = uni(cmd.y), room = uni(cmd.w);
    if (what == HC_EXIT) break;
    uint32_t r0 = 0, r1 = 0, r2 = 0;
    if (what == HC_BEST_HOST) {
      bool idle;
      r0 = best_host_part(c, now, g, room, idle);
      r1 = idle ? 1u : 0u;
    } else if (what == HC_EARLIEST_IDLE) {
      int32_t capped;
      r0 = (uint32_t)earliest_idle_part(c, g, room, capped);
      r1 = (uint32_t)capped;
    } else if (what == HC_PLACE) {
      if (c.nw == MAX_WAVES) place_part<NBOS_MAX_HOSTS / WAVE / MAX_WAVES>(c, now, room, r0, r1, r2);
      else place_part<NBOS_MAX_HOSTS / WAVE>(c, now, room, r0, r1, r2);
    } else {
      int A, Z;
      tick_part(c, now, A, Z, r2);
      r0 = (uint32_t)A; r1 = (uint32_t)Z;
    }
    if (c.lane == 0) { c.m.mail[8 + 4 * c.wid] = (int)r0; c.m.mail[9 + 4 * c.wid] = (int)r1; c.m.mail[10 + 4 * c.wid] = (int)r2; }
    __syncthreads();
  }
}

template <uint32_t F>
__device__ __forceinline__ void tick(Ctx<F> &c, Regs &r, int32_t now) {
  wave_sync();
  const bool autoscale = (c.flags() & NBOS_F_AUTOSCALE) != 0;
  helpers_go(c, HC_TICK, now, 0, 0);
  int A, Z;
  uint32_t sum_c;
  tick_part(c, now, A, Z, sum_c);
  helpers_done(c);
  for (int w = 1; w < c.nw; w++) {
    A += (int)helper_result(c, w, 0);
    Z += (int)helper_result(c, w, 1);
    sum_c += helper_result(c, w, 2);
  }
  int released = 0;
  if (autoscale) {
    // expected capacity f * sum C in whole hosts plus the scaling buffer; hosts being provisioned
    // count as capacity
    const uint32_t per_host = 1000u * (uint32_t)c.p.G;
    const int want = (int)(((uint32_t)c.p.f_milli * sum_c + per_host - 1u) / per_host) + c.p.buffer;
    int n_on = c.n_on;
    const int before = n_on;
    while (n_on < want && n_on < c.p.Hmax) {
      const int h = boot_host(c, r, now, 0u);
      n_on++;
      decide(c, r, now, NBOS_D_SCALE_AUTO, 0, 0, (uint32_t)h);
    }
    if (n_on != before) c32_max(c.m, c.lane, CS_PEAK, (uint32_t)n_on);
    if (c.flags() & NBOS_F_SCALE_IN) {
      while (n_on > want && Z > 0 && A > c.p.min_hosts && released < 2) {
        release_host(c, r, now);
        n_on--; A--; Z--; released++;
      }
    }
    return;
  }
  // without the capacity test: release at most two hosts while too large a share of them is empty
  while ((int64_t)Z * 100 > (int64_t)A * c.p.idle_pct && A > c.p.min_hosts && released < 2) {
    release_host(c, r, now);
    A--; Z--; released++;
  }
}

template <uint32_t F>
__device__ __forceinline__ void on_session_end(Ctx<F> &c, Regs &r, uint32_t s, uint32_t hw, int32_t tm, uint32_t fl,
                                               int32_t now) {
  const uint32_t st = fl & 7u;
  if ((st != SS_PLACED && st != SS_QUEUED) || (fl & SF_ENDING)) return;
  const int g = (int)((fl >> 3) & 7u) + 1;
  c32_add(c.m, c.lane, CS_OPENG, (uint32_t)-g);         // the Reservation lifetime closes at the END event
  c64_add(c.m, c.lane, CL_RESV, (int64_t)g * now);
  if (st == SS_PLACED && tm <= now) {
    end_session(c, r, s, hw, fl, now);
  } else {
    sess_write_flag(c, r, s, fl | SF_ENDING);
    if (st == SS_PLACED) timer_push(c, r, tm, QK_END, s, 0);
  }
}

// ---- retries that fail again, looked at ahead of time (open loop) -----------------------------------
// A retry of a queued cell (Section 3.2.3) that fails once more changes nothing but the session's retry
// count and the time of its timer. Whether it fails is known early: (a) its election fails at the timer's
// time if none of the session's hosts has g idle GPUs then, on the busy-until times as they stand: whatever
// is bound before the timer fires only takes idle GPUs away; (b) no migration target exists before the
// stored bound of c.fu / c.fc; (c) no host can be added while the cluster is at its maximum. (a) is worked
// out here for all sorted timers at once, lane = timer, and stays true; (b) and (c) are tests of uniform
// values when the timer fires. Such a retry then costs a few instructions, and, since it touches nothing
// that an election reads, the event-parallel rounds need not stop at it (retry_horizon).
template <uint32_t F>
__device__ __forceinline__ void retry_lookahead(Ctx<F> &c, const Regs &r) {
  wave_sync();
  const int G = c.p.G;
  const bool cand = c.lane < r.q_n && (c.qk >> 16) == QK_RETRY && !((uint32_t)c.qd & QD_LOOKED);
  if (cand) {
    const SessRec rec = c.m.sess[c.qk & 0xFFFFu];
    const uint32_t hw = (uint32_t)rec.x, fl = (uint32_t)rec.z;
    const int g = (int)((fl >> 3) & 7u) + 1;
    const int32_t vt = c.qt;
    const uint32_t h0 = hw & 1023u, h1 = (hw >> 10) & 1023u, h2 = (hw >> 20) & 1023u;
    const int C0 = committed(c, (int)h0, vt), C1 = committed(c, (int)h1, vt), C2 = committed(c, (int)h2, vt);
    const bool can = (c.m.ready_at[h0] <= vt && C0 + g <= G) || (c.m.ready_at[h1] <= vt && C1 + g <= G) ||
                     (c.m.ready_at[h2] <= vt && C2 + g <= G);
    const bool more = (int)((fl >> 8) & 15u) < c.p.max_retries;        // not the retry that gives the cell up
    uint32_t d = (uint32_t)c.qd | QD_LOOKED;
    if (!can && more) d |= QD_EFAIL | ((uint32_t)(g - 1) << QD_G_SHIFT);
    c.qd = (int32_t)d;
  }
}

// hosts can be added right now (a failed election then gets a host instead of a place in the queue)
template <uint32_t F>
__device__ __forceinline__ bool can_grow(const Ctx<F> &c) {
  return (c.flags() & NBOS_F_SCALE_OUT) && c.n_on < c.p.Hmax;
}

// per lane = sorted timer: it is a retry that is known to fail quietly if it fires now
template <uint32_t F>
__device__ __forceinline__ bool retry_is_quiet(const Ctx<F> &c, const Regs &r) {
  const uint32_t d = (uint32_t)c.qd;
  const int32_t bound_own = c.fu > c.fc ? c.fu : c.fc;                  // lane g-1: no target before this time
  const int32_t bound = __builtin_amdgcn_ds_bpermute((int)((d >> QD_G_SHIFT) & 7u) << 2, bound_own);
  return c.lane < r.q_n && (c.qk >> 16) == QK_RETRY && (d & QD_EFAIL) != 0 &&
         (!(c.flags() & NBOS_F_MIGRATE) || c.qt < bound);
}

// Up to which time a run of arrivals may be evaluated without looking at the timers: the time of the first
// sorted timer that is not a quietly failing retry (or of whatever waits outside the registers), and not
// beyond the time at which the earliest of the quiet ones comes back (one retry interval later).
template <uint32_t F>
__device__ __forceinline__ int32_t retry_horizon(Ctx<F> &c, const Regs &r, int32_t until) {
  if (r.q_n == 0) return r.q_head_t;
  if (((uint32_t)lane_get((int)c.qk, 0) >> 16) != QK_RETRY) return r.q_head_t;
  if (can_grow(c)) return r.q_head_t;
  // retries due up to `until` that have not been looked at yet
  if (wballot(c.lane < r.q_n && (c.qk >> 16) == QK_RETRY && !((uint32_t)c.qd & QD_LOOKED) && c.qt <= until) != 0)
    retry_lookahead(c, r);
  const uint64_t loud = wballot(c.lane < r.q_n && !retry_is_quiet(c, r));
  const int first = loud != 0 ? (int)__builtin_ctzll(loud) : r.q_n;
  if (first == 0) return r.q_head_t;
  int32_t lim = first < r.q_n ? lane_get(c.qt, first) : (r.o_n > 0 ? r.o_min_t : NEVER);
  const int64_t back = (int64_t)r.q_head_t + c.p.retry_iv;
  if (back < lim) lim = (int32_t)back;
  return lim;
}

// The due timers at the head of the sorted registers that are retries known to fail quietly - all of them up
// to the first timer that is not, "due" meaning at or before t_limit - fire at once, lane = timer: each
// counts its retry in its session's record and moves one retry interval on. The timers that are then no
// longer earlier than everything that waits in the session records go there; the others are merged back
// into the sorted registers (both parts are sorted already: a timer's new place is its rank in its own part
// plus the number of timers of the other part before it). queued_lanes: lanes of the current tile whose
// prefetched record showed a queued session (the records of the retries fired here are among those, or
// stale already). Returns false if the earliest timer is no such retry (nothing but the marks of
// retry_lookahead is changed then).
template <uint32_t F>
__device__ __forceinline__ bool fire_quiet_retries(Ctx<F> &c, Regs &r, int32_t t_limit, uint64_t queued_lanes) {
  if (((uint32_t)lane_get((int)c.qk, 0) >> 16) != QK_RETRY) return false;
  if (wballot(c.lane < r.q_n && (c.qk >> 16) == QK_RETRY && !((uint32_t)c.qd & QD_LOOKED) && c.qt <= t_limit) != 0)
    retry_lookahead(c, r);
  if (!((uint32_t)lane_get(c.qd, 0) & QD_EFAIL)) return false;
  if (can_grow(c)) return false;
  const uint64_t loud = ~wballot(retry_is_quiet(c, r) && c.qt <= t_limit);
  const int n = loud != 0 ? (int)__builtin_ctzll(loud) : WAVE;        // (quiet timers are below q_n)
  if (n == 0) return false;
  const bool mine = c.lane < n;
  const int32_t last = lane_get(c.qt, n - 1);
  r.t_end = r.t_end > last ? r.t_end : last;
  r.dirty |= queued_lanes;
  wave_sync();
  const uint32_t s = c.qk & 0xFFFFu;
  int32_t nt = c.qt;
  bool far = false;
  if (mine) {
    const uint32_t fl = (uint32_t)c.m.sess[s].z;
    const int retries = (int)((fl >> 8) & 15u) + 1;                    // below max_retries before: see retry_lookahead
    nt = c.m.sess[s].y + retries * c.p.retry_iv;
    far = r.o_n > 0 && !(nt < r.o_min_t || (nt == r.o_min_t && c.qk < r.o_min_k));
    uint32_t nfl = (fl & ~(15u << 8)) | ((uint32_t)retries << 8);
    if (far) {
      nfl = (nfl & ~(3u << CL_KIND_SHIFT)) | (QK_RETRY << CL_KIND_SHIFT);
      c.m.due[s] = nt;
      c.ovf_dur[s] = c.qd & QD_DUR_MASK;
    }
    c.m.sess[s].z = (int)nfl;
  }
  const uint64_t far_m = wballot(far);
  const uint64_t near_m = wballot(mine && !far);
  const bool kept = c.lane >= n && c.lane < r.q_n;
  r.o_n += __builtin_popcountll(far_m);
  // merge: the timers that stay where they are (kept) and those that moved on inside the registers (near)
  int pos = kept ? c.lane - n : lane_rank(near_m);
  for (uint64_t w = near_m; w != 0; w &= w - 1) {
    const int j = (int)__builtin_ctzll(w);
    const int32_t tj = lane_get(nt, j);
    const uint32_t kj = (uint32_t)lane_get((int)c.qk, j);
    const bool before_j = c.qt < tj || (c.qt == tj && c.qk < kj);     // (kept lanes: their own key)
    const int kept_before = __builtin_popcountll(wballot(kept && before_j));
    if (kept && !before_j) pos++;
    if (c.lane == j) pos += kept_before;
  }
  const int alive = r.q_n - __builtin_popcountll(far_m);
  const bool dead = !(kept || (mine && !far));
  if (dead) pos = alive + lane_rank(wballot(dead));
  const int32_t vt = dead ? NEVER : nt;
  const int32_t vd = dead ? 0 : (mine ? (c.qd & QD_DUR_MASK) : c.qd);
  const uint32_t vk = dead ? 0xFFFFFFFFu : c.qk;
  c.qt = __builtin_amdgcn_ds_permute(pos << 2, vt);
  c.qd = __builtin_amdgcn_ds_permute(pos << 2, vd);
  c.qk = (uint32_t)__builtin_amdgcn_ds_permute(pos << 2, (int)vk);
  r.q_n = alive;
  if (r.q_n == 0 && r.o_n > 0) refill(c, r);
  r.q_head_t = r.q_n > 0 ? lane_get(c.qt, 0) : NEVER;
  return true;
}

// ---- one event-parallel round over the lanes in `run` (see the file header) -----------------------
// Returns the mask of lanes whose cells were started. rec = the lane's prefetched session record.
// next_lost: the lane after the started ones lost its election (another round would start nothing there).
template <uint32_t F>
__device__ __forceinline__ uint64_t batch_round(Ctx<F> &c, Regs &r, uint64_t run, int32_t vt, int32_t vd, uint32_t sid,
                                                const SessRec &rec, bool &next_lost) {
  wave_sync();
  const int G = c.p.G;
  const bool in_run = (run >> c.lane) & 1u;
  const uint32_t hw = (uint32_t)rec.x, fl = (uint32_t)rec.z;
  const int g = (int)((fl >> 3) & 7u) + 1;
  const uint32_t h0 = hw & 1023u, h1 = (hw >> 10) & 1023u, h2 = (hw >> 20) & 1023u;
  // committed GPUs of the three hosts at this lane's own time
  const int4 a0 = c.m.fin[2 * h0], b0 = c.m.fin[2 * h0 + 1];
  const int4 a1 = c.m.fin[2 * h1], b1 = c.m.fin[2 * h1 + 1];
  const int4 a2 = c.m.fin[2 * h2], b2 = c.m.fin[2 * h2 + 1];
  const int32_t r0 = c.m.ready_at[h0], r1 = c.m.ready_at[h1], r2 = c.m.ready_at[h2];
  const int C0 = (a0.x > vt) + (a0.y > vt) + (a0.z > vt) + (a0.w > vt) + (b0.x > vt) + (b0.y > vt) + (b0.z > vt) + (b0.w > vt);
  const int C1 = (a1.x > vt) + (a1.y > vt) + (a1.z > vt) + (a1.w > vt) + (b1.x > vt) + (b1.y > vt) + (b1.z > vt) + (b1.w > vt);
  const int C2 = (a2.x > vt) + (a2.y > vt) + (a2.z > vt) + (a2.w > vt) + (b2.x > vt) + (b2.y > vt) + (b2.z > vt) + (b2.w > vt);
  const uint32_t k0 = (r0 <= vt && C0 + g <= G) ? (((uint32_t)C0 << 12) | (h0 << 2) | 0u) : 0xFFFFFFFFu;
  const uint32_t k1 = (r1 <= vt && C1 + g <= G) ? (((uint32_t)C1 << 12) | (h1 << 2) | 1u) : 0xFFFFFFFFu;
  const uint32_t k2 = (r2 <= vt && C2 + g <= G) ? (((uint32_t)C2 << 12) | (h2 << 2) | 2u) : 0xFFFFFFFFu;
  uint32_t kb = umin(k0, umin(k1, k2));
  if (c.flags() & NBOS_F_STICKY_EXECUTOR) {
    const uint32_t last = hw >> 30;
    const uint32_t kp = last == 1u ? k0 : (last == 2u ? k1 : (last == 3u ? k2 : 0xFFFFFFFFu));
    if (kp != 0xFFFFFFFFu) kb = kp;
  }
  const bool won = in_run && kb != 0xFFFFFFFFu;
  const int lead = (int)(kb & 3u);
  const int ch = won ? (int)((kb >> 2) & 1023u) : 0;
  // who binds where: the lowest lane that chose a host marks it
  if (won) atomicMin(&c.m.mark[ch], c.lane);
  wave_sync();
  const int32_t first = c.m.mark[ch];        // the lowest lane that binds on the host this lane chose
  wave_sync();
  if (won) c.m.mark[ch] = MARK_FREE;
  const uint64_t lost = run & wballot(in_run && !won);
  const uint64_t bad = lost | (run & wballot(in_run && first < c.lane));
  const uint64_t below = bad ? ((1ull << __builtin_ctzll(bad)) - 1ull) : ~0ull;
  next_lost = bad != 0 && ((lost >> __builtin_ctzll(bad)) & 1u) != 0;     // the lane that ends the prefix lost its election
  const uint64_t done = run & below;
  if (__builtin_expect(done == 0, 0)) return 0;
  const bool mine = (done >> c.lane) & 1u;
  const int32_t finish = vt + vd;
  if (mine) {
    // bind g free GPUs of the chosen host: rewrite its row
    int4 a = lead == 0 ? a0 : (lead == 1 ? a1 : a2);
    int4 b = lead == 0 ? b0 : (lead == 1 ? b1 : b2);
    int need = g;
    if (need > 0 && a.x <= vt) { a.x = finish; need--; }
    if (need > 0 && G > 1 && a.y <= vt) { a.y = finish; need--; }
    if (need > 0 && G > 2 && a.z <= vt) { a.z = finish; need--; }
    if (need > 0 && G > 3 && a.w <= vt) { a.w = finish; need--; }
    if (need > 0 && G > 4 && b.x <= vt) { b.x = finish; need--; }
    if (need > 0 && G > 5 && b.y <= vt) { b.y = finish; need--; }
    if (need > 0 && G > 6 && b.z <= vt) { b.z = finish; need--; }
    if (need > 0 && G > 7 && b.w <= vt) { b.w = finish; need--; }
    c.m.fin[2 * ch] = a; c.m.fin[2 * ch + 1] = b;
    const uint32_t nhw = (hw & 0x3FFFFFFFu) | ((uint32_t)(lead + 1) << 30);
    c.m.sess[sid].x = (int)nhw; c.m.sess[sid].y = finish;
  }
  // counters over the started lanes: order-free sums go to LDS accumulators (one ds_add per lane)
  const uint32_t n = (uint32_t)__builtin_popcountll(done);
  r.c_started += n; r.c_imm += n; r.h0 += n;
  r.reused += (uint32_t)__builtin_popcountll(wballot(mine && (hw >> 30) == (uint32_t)lead + 1u));
  if (mine) {
    atomicAdd(&c.m.c64[CL_BDUR], (unsigned long long)(uint32_t)vd);
    atomicAdd(&c.m.c64[CL_BGEXEC], (unsigned long long)(uint32_t)(g * vd));
    atomicMax(&c.m.c32[CS_BLAZY], (uint32_t)finish);
  }
  // digest: d * P^n + sum over started lanes of code * P^(n - 1 - rank), the sum in three limbs
  const int rank = lane_rank(done);
  const uint64_t code = decision_code(vt, NBOS_D_START, sid, (uint32_t)lead, (uint32_t)ch);
  // the terms are added up by the LDS unit, in the spare slot behind the table of powers
  wave_sync();
  if (c.lane == 0) c.m.ppow[65] = 0;
  if (mine) atomicAdd(&c.m.ppow[65], (unsigned long long)(code * c.m.ppow[n - 1u - (uint32_t)rank]));
  wave_sync();
  const unsigned long long sm = c.m.ppow[65];
  const uint64_t sum = (uint64_t)uni((uint32_t)sm) | ((uint64_t)uni((uint32_t)(sm >> 32)) << 32);
  const unsigned long long pn = c.m.ppow[n];
  const uint64_t pnu = (uint64_t)uni((uint32_t)pn) | ((uint64_t)uni((uint32_t)(pn >> 32)) << 32);
  r.digest = r.digest * pnu + sum;
  if (__builtin_expect(c.dlog != nullptr, 0)) {
    const int64_t at = (int64_t)r.n_dec + rank;
    if (mine && at < c.p.dlog_stride) c.dlog[at] = code;
  }
  r.n_dec += n;
  return done;
}

// ---- LDS layout of one replay and its initial state (S0) -------------------------------------------
template <bool CL>
__device__ __forceinline__ Lds lds_carve(const KParams &p, unsigned char *q) {
  Lds m;
  m.c64 = (unsigned long long *)q;  q += 8 * 8;
  m.c32 = (uint32_t *)q;            q += 16 * 4;
  m.hist = (uint32_t *)q;           q += 32 * 4;
  m.ppow = (unsigned long long *)q; q += 66 * 8;
  m.mail = (int32_t *)q;            q += MAIL_WORDS * 4;
  m.fin = (int4 *)q;                q += (size_t)p.HP * 32;
  m.ready_at = (int32_t *)q;        q += (size_t)p.HP * 4;
  m.mark = (int32_t *)q;            q += (size_t)p.HP * 4;
  m.hsn = (uint32_t *)q;            q += (size_t)p.HP * 4;
  m.warm = (int32_t *)q;            q += p.warm_n > 0 ? (size_t)p.HP * 16 : 0;
  // 16-byte aligned: the refill reads four times at once
  m.due = (int32_t *)q;             q += (size_t)((p.n_cap + 3) / 4 * 4) * 4;
  m.stage = (int32_t *)q;           q += WAVE * 4;
  m.sess = (SessRec *)q;
  return m;
}

// hosts 0..H0-1 ready at time 0, the rest off; sessions unplaced (all threads of the workgroup take part)
template <bool CL>
__device__ __forceinline__ void lds_init(const KParams &p, const Lds &m, int s_lo, int n_sess) {
  const int tid = threadIdx.x, nt = blockDim.x;
  if (tid < 8) m.c64[tid] = 0;
  if (tid < 16) m.c32[tid] = tid == CS_NON || tid == CS_PEAK ? (uint32_t)p.H0 : 0u;
  if (tid < 32) m.hist[tid] = 0;
  if (tid < MAIL_WORDS) m.mail[tid] = 0;
  if (tid == 0) {
    unsigned long long pw = 1;
    for (int i = 0; i <= 64; i++) { m.ppow[i] = pw; pw *= DIGEST_PRIME; }
  }
  for (int i = tid; i < 2 * p.HP; i += nt) m.fin[i] = make_int4(0, 0, 0, 0);
  for (int h = tid; h < p.HP; h += nt) {
    m.ready_at[h] = h < p.H0 ? 0 : NEVER;
    m.mark[h] = MARK_FREE;
    m.hsn[h] = 0;
  }
  if (p.warm_n > 0) {
    for (int i = tid; i < 4 * p.HP; i += nt) m.warm[i] = 0;     // initial hosts: warm from time 0
  }
  for (int s = tid; s < n_sess; s += nt) {
    const uint32_t g = p.sess_gpus[s_lo + s];
    m.sess[s].x = 0; m.sess[s].y = 0; m.sess[s].z = (int)(SS_UNPLACED | ((g - 1u) << 3));
  }
  for (int s = tid; s < (p.n_cap + 3) / 4 * 4; s += nt) m.due[s] = NEVER;
  __syncthreads();
}

// ---- S10: close the integrals at t_end and write the result record ---------------------------------
__device__ __forceinline__ void write_stats(const KParams &p, const Lds &m, const Regs &r, int rep) {
  __syncthreads();                          // every wave of the workgroup comes here; wave 0 holds the results
  const int lane = threadIdx.x;
  const int32_t t_end = r.t_end > r.lazy_max ? r.t_end : r.lazy_max;
  nbos_stats *out = p.stats + rep;
  if (lane < 32) out->delay_hist[lane] = m.hist[lane] + (lane == 0 ? r.h0 : 0u);
  if (lane == 0) {
    const int64_t sum_delay = (int64_t)m.c64[CL_SUMDELAY], g_wait = (int64_t)m.c64[CL_GWAIT];
    out->status = r.status; out->n_decisions = r.n_dec;
    out->sessions_placed = m.c32[CS_PLACED]; out->sessions_rejected = m.c32[CS_REJECTED];
    out->cells_total = r.c_total; out->cells_immediate = r.c_imm; out->cells_started = r.c_started;
    out->cells_queued = m.c32[CS_QUEUED]; out->cells_aborted = m.c32[CS_ABORTED];
    out->cells_dropped_busy = r.c_busy; out->cells_dropped_unplaced = r.c_unplaced;
    out->executor_reused = r.reused; out->migrations = m.c32[CS_MIGR];
    out->scale_out_hosts = m.c32[CS_SO]; out->scale_in_hosts = m.c32[CS_SI]; out->peak_hosts = m.c32[CS_PEAK];
    out->migrations_warm = m.c32[CS_MIGRWARM];
    out->max_delay_ms = (int32_t)m.c32[CS_MAXDELAY]; out->t_end_ms = t_end;
    const int64_t sum_dur = r.sum_dur + (int64_t)m.c64[CL_BDUR], g_exec = r.g_exec + (int64_t)m.c64[CL_BGEXEC];
    out->sum_delay_ms = sum_delay; out->sum_tct_ms = sum_dur + sum_delay;
    out->gpu_ms_executed = g_exec; out->gpu_ms_committed = g_exec + g_wait;
    out->gpu_ms_provisioned = (int64_t)m.c64[CL_PROV] + (int64_t)m.c32[CS_NON] * p.G * t_end;
    out->reservation_gpu_ms = (int64_t)m.c64[CL_RESV] + (int64_t)(int32_t)m.c32[CS_OPENG] * t_end;
    out->sub_gpu_ms = (int64_t)m.c64[CL_SUB] + (int64_t)(int32_t)m.c32[CS_SUMS] * t_end;
    out->replica_ms = (int64_t)m.c64[CL_REPL] + (int64_t)(int32_t)m.c32[CS_NREP] * t_end;
    out->digest = r.digest;
  }
}

template <uint32_t F>
__global__ void __launch_bounds__(MAX_WAVES * WAVE) nbos_replay_lds_kernel(KParams p) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int rep = launch_slot_replay(p);
  const int lane = threadIdx.x & (WAVE - 1);
  if (rep >= p.n_replays) return;

  const int trace = p.trace_of_replay[rep];
  const int64_t ev_lo = p.ev_offset[trace], ev_hi = p.ev_offset[trace + 1];
  const int s_lo = p.sess_offset[trace];
  const int n_sess = p.sess_offset[trace + 1] - s_lo;

  const Lds m = lds_carve<false>(p, lds_raw);
  lds_init<false>(p, m, s_lo, n_sess);
  PROF_BEGIN();

  const int32_t caplim = p.cap_milli[rep] * p.G * 3;
  Ctx<F> c{p, m, lane, caplim / 1000, p.dlog ? p.dlog + (int64_t)rep * p.dlog_stride : nullptr,
        NEVER, 0, 0xFFFFFFFFu, 0xFFFFFFFFu, 0};
  c.n_sess = n_sess;
  c.ovf_dur = p.ovf_dur + (int64_t)rep * p.n_cap;
  c.nw = (int)(blockDim.x / WAVE);
  c.wid = (int)(threadIdx.x / WAVE);
  c.dyn = dynamic_limit_matters(p, c.flags(), c.slim);
  c.n_on = p.H0;
  Regs r;
  memset(&r, 0, sizeof r);
  r.digest = 0xCBF29CE484222325ULL;
  r.q_head_t = NEVER;
  r.o_min_t = NEVER;
  r.min_s = -1;
  r.cl_win = 1024;
  if (c.wid != 0) {
    helper_loop(c);
  } else {

  const bool ticking = (c.flags() & (NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE)) != 0;
  const bool batching = p.batch != 0;
  // Retries are looked at ahead of time (retry_lookahead) unless the cap moves with the cluster's sums: then
  // no bound on the next migration target is kept and hardly any retry is known to fail
  const bool look_ahead = !((c.flags() & NBOS_F_DYNAMIC_SR) && c.dyn);
  // hash buckets (power of two <= HP) for spotting two events of one session in a tile
  const uint32_t dup_mask = (1u << (31 - __builtin_clz((uint32_t)p.HP))) - 1u;
  int32_t tick_t = ticking ? p.scale_iv : NEVER;
  int32_t due_t = tick_t;                   // earliest queued timer or auto-scaler period
  int cooldown = 0;                         // serial items to go before the next parallel round

  // S1: stream the events, one per lane per tile, next tile in flight
  int64_t base = ev_lo;                     // first event of the tile held in (nt, nd, ns)
  int32_t vt = 0, vd = 0, vs = 0, nt = 0, nd = 0, ns = 0;
  if (base + lane < ev_hi) { nt = p.ev_time[base + lane]; nd = p.ev_dur[base + lane]; ns = p.ev_sk[base + lane]; }

  bool final = false;
  while (r.status == NBOS_OK) {
    SessRec rec = {0, 0, 0};                // prefetched session record of this lane's event
    bool fast = false;                      // this lane's event is a cell of an idle placed session
    uint64_t todo = 0;
    uint32_t sid = 0;
    int32_t last_t = 0;                     // time of the tile's last event
    if (base < ev_hi) {
      vt = nt; vd = nd; vs = ns;
      const int64_t cur = base;
      last_t = lane_get(vt, (int)(ev_hi - cur < WAVE ? ev_hi - cur - 1 : WAVE - 1));
      base += WAVE;
      if (base + lane < ev_hi) { nt = p.ev_time[base + lane]; nd = p.ev_dur[base + lane]; ns = p.ev_sk[base + lane]; }
      const bool valid = cur + lane < ev_hi;
      const bool is_last = cur + lane == ev_hi - 1;
      sid = valid ? ((uint32_t)vs & 0xFFFFFFu) : 0u;
      const bool is_cell = ((uint32_t)vs >> 24) == NBOS_EV_CELL;
      c.vsid = valid ? sid : 0xFFFFFFFFu;
      wave_sync();
      if (valid) rec = m.sess[sid];
      // Cells of sessions in a final state (rejected / ended) and cells that arrive while the
      // session's running cell lasts beyond them change nothing: count them, skip them. Neither
      // condition can be undone before the event's time. The last event of the trace is never
      // skipped, so timers due before it still run first.
      const uint32_t st = (uint32_t)rec.z & 7u;
      const bool dead = st == SS_REJECTED || st == SS_ENDED;
      const bool running = st == SS_PLACED && rec.y > vt;
      const bool skip = valid && !is_last && (dead || (is_cell && running));
      r.c_total += (uint32_t)__builtin_popcountll(wballot(valid && is_cell));
      r.c_unplaced += (uint32_t)__builtin_popcountll(wballot(skip && is_cell && dead));
      r.c_busy += (uint32_t)__builtin_popcountll(wballot(skip && is_cell && !dead));
      fast = valid && is_cell && st == SS_PLACED && !running && !((uint32_t)rec.z & SF_ENDING);
      todo = wballot(valid && !skip);
      r.dirty = 0;
      if (batching) {
        // a lane whose session may also belong to an earlier lane of the tile keeps out of the rounds
        const uint32_t b = sid & dup_mask;
        if (valid) atomicMin(&m.mark[b], lane);
        wave_sync();
        const bool dup = valid && m.mark[b] < lane;
        wave_sync();
        if (valid) m.mark[b] = MARK_FREE;
        // the buckets are few (a lane in eight shares one with an earlier lane by chance): keep only the
        // lanes that really have their session in an earlier lane
        for (uint64_t w = wballot(dup); w != 0; w &= w - 1) {
          const int j = (int)__builtin_ctzll(w);
          const uint32_t sj = (uint32_t)lane_get((int)sid, j);
          if (wballot(valid && sid == sj && lane < j) != 0) r.dirty |= 1ull << j;
        }
      }
      if (ev_hi - cur <= WAVE) {
        int32_t tl = lane_get(vt, (int)(ev_hi - cur - 1));
        r.t_end = r.t_end > tl ? r.t_end : tl;
      }
    } else {
      final = true;
      wave_sync();
      const int32_t bl = (int32_t)uni(m.c32[CS_BLAZY]);       // finish times bound by the rounds
      r.lazy_max = r.lazy_max > bl ? r.lazy_max : bl;
    }
    const uint64_t fastmask = wballot(fast);
    PROF(PC_TILE, 1);
    const uint64_t queued_lanes = wballot(((uint32_t)rec.z & 7u) == SS_QUEUED);
    bool hz_known = false;
    int32_t hz = 0;
    for (;;) {
      if (__builtin_expect(r.status != NBOS_OK, 0)) break;
      int i = 0;
      int32_t t = NEVER;
      if (todo != 0) { i = (int)__builtin_ctzll(todo); t = lane_get(vt, i); }
      else if (!final) break;
      wave_sync();
      uint32_t a_s, a_hw, a_fl;
      int32_t a_now, a_sub, a_dur;
      [[maybe_unused]] bool is_retry = false;      // (path profile)
      bool hz_kept = false;
      if (__builtin_expect(t < due_t, 1)) {
        const uint64_t bit = 1ull << i;
        const uint64_t clean = fastmask & ~r.dirty;
        if (__builtin_expect(batching && cooldown == 0 && (clean & bit) != 0, 1)) {
          // ---- event-parallel round over the run of fast arrivals that starts at lane i ----
          // the run may go on past retries that are known to fail quietly
          int32_t run_due = due_t;
          if (look_ahead && due_t == r.q_head_t && due_t <= last_t) {
            if (!hz_known) { PROF(PC_LOOP_HORIZON, 1); hz = retry_horizon(c, r, last_t); hz_known = true; PROF(PC_HORIZON, 1); }    // (rounds change nothing it looks at)
            run_due = hz < tick_t ? hz : tick_t;
          }
          const uint64_t eligible = clean & wballot(vt < run_due);
          const uint64_t blockers = todo & ~eligible;
          const uint64_t run = blockers ? (todo & ((1ull << __builtin_ctzll(blockers)) - 1ull)) : todo;
          if (__builtin_expect((run & (run - 1)) != 0, 1)) {          // at least two lanes
            bool next_lost;
            PROF(PC_LOOP_ROUND, 1);
            const uint64_t done = batch_round(c, r, run, vt, vd, sid, rec, next_lost);
            PROF(PC_ROUND, __builtin_popcountll(done));
            // none or one started, or the next arrival has just lost its election: it goes alone
            cooldown = ((done & (done - 1)) == 0 || next_lost) ? 1 : 0;
            if (__builtin_expect(done != 0, 1)) { todo &= ~done; continue; }
          }
        }
        if (cooldown > 0) cooldown--;
        // ---- arrival i, serial ----
        hz_kept = hz_known;                   // (the attempt below says whether the horizon is still good)
        hz_known = false;
        todo &= ~bit;
        const uint32_t sk = (uint32_t)lane_get(vs, i);
        const uint32_t s = sk & 0xFFFFFFu;
        if (__builtin_expect((clean & bit) != 0, 1)) {
          a_s = s; a_hw = (uint32_t)lane_get(rec.x, i);
          a_fl = (uint32_t)lane_get(rec.z, i);
          a_now = t; a_sub = t; a_dur = lane_get(vd, i);
        } else {
          const uint32_t kind = sk >> 24;
          uint32_t hw, fl;
          int32_t tm;
          if ((r.dirty >> i) & 1u) {
            const SessRec cur = m.sess[s];
            hw = uni((uint32_t)cur.x); tm = uni(cur.y); fl = uni((uint32_t)cur.z);
          } else {
            hw = (uint32_t)lane_get(rec.x, i); tm = lane_get(rec.y, i); fl = (uint32_t)lane_get(rec.z, i);
          }
          if (kind == NBOS_EV_CELL) {           // S4-S8 (counted in c_total at tile load)
            const uint32_t st = fl & 7u;
            if (st == SS_PLACED && tm <= t) {
              a_s = s; a_hw = hw; a_fl = fl & ~(SF_QONCE | (15u << 8)); a_now = t; a_sub = t; a_dur = lane_get(vd, i);
            } else {
              if (st == SS_PLACED || st == SS_QUEUED) r.c_busy++; else r.c_unplaced++;
              PROF(PC_DROP, 1);
              continue;
            }
          } else {
            PROF(PC_LOOP_STARTEND, 1);
            if (kind == NBOS_EV_START) { session_start(c, r, s, fl, t); PROF(PC_START, 1); }      // S3, S7
            else { on_session_end(c, r, s, hw, tm, fl, t); PROF(PC_END, 1); }
            due_t = r.q_head_t < tick_t ? r.q_head_t : tick_t;
            continue;
          }
        }
      } else {
        // ---- a timer may be due (S2); always taken while draining ----
        PROF(PC_LOOP_TIMER, 1);
        hz_known = false;
        bool fire_q = r.q_n > 0, fire_t = ticking;
        if (final) {
          if (fire_t) fire_t = fire_q ? tick_t < r.q_head_t : tick_t < r.lazy_max;
          if (fire_t) fire_q = false;
        } else {
          if (fire_q) fire_q = r.q_head_t <= t;
          if (fire_t) fire_t = tick_t <= t;
          if (fire_q && fire_t) { if (r.q_head_t <= tick_t) fire_t = false; else fire_q = false; }
        }
        if (__builtin_expect(fire_t, 0)) {
          tick(c, r, tick_t);
          tick_t += p.scale_iv;
          due_t = r.q_head_t < tick_t ? r.q_head_t : tick_t;
          PROF(PC_TICK, 1);
          continue;
        }
        if (__builtin_expect(!fire_q, 0)) break;   // only reached while draining: nothing is left
        // (timers fire up to the next arrival, and up to the next auto-scaler period: that one runs after the
        // timers of its own instant and before all later ones)
        if (look_ahead && fire_quiet_retries(c, r, t < tick_t ? t : tick_t, queued_lanes)) {
          PROF(PC_QUIET_RETRIES, 1);
          due_t = r.q_head_t < tick_t ? r.q_head_t : tick_t;
          continue;
        }
        const int32_t now = r.q_head_t;
        const uint32_t key = (uint32_t)lane_get((int)c.qk, 0);
        const int32_t dur = lane_get(c.qd, 0) & QD_DUR_MASK;
        const uint32_t s = key & 0xFFFFu;
        const SessRec cur = m.sess[s];        // (asked for before the pop, which does not touch this record)
        timer_pop(c, r);
        r.t_end = r.t_end > now ? r.t_end : now;
        const uint32_t hw = uni((uint32_t)cur.x), fl = uni((uint32_t)cur.z);
        if ((key >> 16) != QK_RETRY) {
          end_session(c, r, s, hw, fl, now);
          due_t = r.q_head_t < tick_t ? r.q_head_t : tick_t;
          PROF(PC_TIMER_OTHER, 1);
          continue;
        }
        a_s = s; a_hw = hw; a_fl = fl; a_now = now; a_sub = uni(cur.y); a_dur = dur;
        is_retry = true;
      }
      PROF(PC_LOOP_ATTEMPT, 1);
      PROF_ATTEMPT_BEGIN(m, r);
      const int32_t did = attempt(c, r, a_s, a_hw, a_fl, a_now, a_sub, a_dur);
      PROF_ATTEMPT_END(m, r, is_retry);
      due_t = r.q_head_t < tick_t ? r.q_head_t : tick_t;
      // an arrival that only bound GPUs, or only joined the queue, leaves the horizon of the rounds as it
      // was (binding keeps quiet retries quiet; the new retry has not been looked at: it ends the horizon)
      if (hz_kept && did >= 0) {
        hz_known = true;
        hz = hz < did ? hz : did;
        if (r.o_n > 0 && r.o_min_t < hz) hz = r.o_min_t;      // (the push may have moved a sorted timer out)
      }
    }
    if (final) break;
  }
  helpers_go(c, HC_EXIT, 0, 0, 0);
  }  // wave 0

  write_stats(p, m, r, rep);
  PROF_OUT(rep);
}

}  // namespace ldsk
}  // namespace
