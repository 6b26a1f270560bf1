// nbos_kernel_reg.hpp — replay kernel for clusters of at most 64 hosts: host state in registers.
//
// One workgroup (one wave64) per replay.
//
// GPUs:   fin[j], j < NJ = ceil(hosts_max / 8). Lane L = (hl = L >> 3, k = L & 7) holds in fin[j] the
//         "busy until" time of GPU k of host 8 j + hl. A GPU is committed at time t iff fin > t, so
//         the ballot of (fin[j] > now) is a 64-bit word with one byte of busy-GPU bits per host.
//         Binding g GPUs for a cell (paper Section 3.3) = writing its finish time into the g lowest
//         free GPUs of the host byte (ballot + lane rank). Completions need no timer: every timer
//         due at or before an item runs before that item and a completion only lowers C, so
//         "released once the clock has passed fin" is exact.
// Hosts:  lane h = host h holds ready_at (0 initial, NEVER while off: provisioning needs no timer
//         either, Section 3.4.2) and S | replicas << 16 (Section 3.4.1). The committed count C of
//         every host in lane = host layout comes from the NJ ballots by a byte extract + popcount.
// Choice: feasibility by ballot; executor election (Section 3.2.2) tests 3 bits of that ballot;
//         placement / migration target = wave minimum of the packed key (C, S, host), so ties go
//         to the lowest host index.
// Events: coalesced dword loads, one event per lane, next tile in flight while the current tile
//         is consumed from registers (v_readlane). At tile start every lane prefetches the record of
//         its event's session from LDS; events of sessions in a final state (rejected / ended) are
//         counted in bulk and skipped. A record written during the tile marks the matching lanes
//         dirty, and only those are read again from LDS.
// Timers: RETRY of a queued cell (Section 3.2.3) and the END of a session that was busy when its END
//         arrived are the only timers that change decisions. The 64 earliest live sorted in
//         registers (insert = ballot + DPP wave shift, pop = DPP wave shift); later ones stay with
//         their session (a flag in its record, their time implied by it) until the registers run empty.
// Closed loop (the paper's section "Interactive Deep Learning Training"; nbos_replay_reg_closed_kernel at the end of this file): only the
//         first STARTs come from the stream, every other event of a session is a timer that is due a
//         think time after the session's previous cell is over. See nbos_kernel_closed.hpp for the
//         chain records this reads and for the same scheme on the any-size kernel.
// Sessions in LDS, 8 bytes each: one word with the state, g, the retry count, the three replica hosts
//         (6 bits each) and the last executor slot; one time word (busy-until, or the submit time while
//         queued). The duration of a queued cell travels with its timer.
#pragma once
#include "nbos_common.hpp"

namespace {
namespace regk {

// Session record: x = state (bits 0-2) | g - 1 (3-5) | ENDING (6) | RK_OVF (7) | retries (8-11) |
// host of slot 0, 1, 2 (6 bits each from bit 12) | last executor slot + 1 (30-31); y = time word.
// The code below calls the word `hw` where it looks at the hosts and `fl` where it looks at the low
// bits; both names hold the whole word.
constexpr uint32_t RK_OVF = 1u << 7;
constexpr uint32_t RK_FLAGS = 0xFFFu;        // the bits below the hosts
__device__ __forceinline__ uint32_t slot_host(uint32_t hw, uint32_t slot) { return (hw >> (12u + 6u * slot)) & 63u; }

struct Lds {
  int32_t *stage;    // [64] sessions whose timers move into the registers
  int32_t *warm;     // [64][4] when each pre-warmed container of a host is available (only with the pool)
  int2 *sess;
  uint32_t *hist;
  uint32_t *c32;
  unsigned long long *c64;
};

// hot uniform registers
struct Regs {
  uint32_t n_dec, c_total, c_imm, c_started, c_busy, c_unplaced, reused, h0;
  int64_t sum_dur, g_exec;
  uint64_t digest;
  int32_t lazy_max, t_end;
  int32_t q_n, q_head_t;                 // sorted register queue: size, time of lane 0
  int32_t o_n, o_min_t;                  // timers outside the registers: how many, the earliest
  uint32_t o_min_k;
  int32_t status;
  uint64_t dirty;                        // lanes of the current tile whose prefetched record is stale
  uint64_t slow_lanes;                   // lanes of the current tile whose prefetched record showed no idle placed session
  // closed loop: the event being handled, its duration and kind (packed as in Ctx::qx), its session's next
  // event and the think time before that; the time window the next refill takes
  int32_t cl_e, cl_x, cl_nx, cl_nth, cl_win;
};

template <int NJ, uint32_t F>
struct Ctx {
  const KParams &p;
  Lds m;
  int lane;
  int n_sess;
  int32_t slim;              // floor(cap_milli * G * 3 / 1000): S + g <= slim is the cap test
  uint64_t *dlog;
  int32_t *ovf_dur;          // [n_sess] durations of queued cells whose timer is outside the registers
  // per-lane state
  int32_t fin[NJ];
  int32_t hr;                // ready_at of host = lane
  uint32_t hs;               // S | nrep << 16 of host = lane
  int32_t qt, qd;            // sorted timers, entry i in lane i
  uint32_t qk;
  uint32_t vsid;             // session id of this lane's event in the current tile (~0 if none)
  int32_t fu;                // lane g-1 (g = 1..8): no host can have g idle GPUs before this time
  // closed loop: the replay's cursors, the events of the trace; and with every sorted timer what firing
  // it needs: qd = the event's index, qx = its duration | kind << 28 | CLX_LOADED (0: not loaded yet),
  // qnx / qnth = its chain record
  int32_t *cl_cur;
  const int32_t *cl_dur, *cl_sk;
  const int2 *cl_chain;
  int32_t qx, qnx, qnth;
  bool dyn;                  // the dynamic limit can differ from the replay's cap (see dynamic_limit_matters)
  static constexpr bool closed = closed_loop_instance(F);
  __device__ __forceinline__ uint32_t flags() const { return instance_flags<F>(p); }
};

// write a session record; lanes of the current tile that prefetched it go stale
template <int NJ, uint32_t F>
__device__ __forceinline__ void sess_write(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t hw, int32_t tm, uint32_t fl) {
  if (c.lane == 0) c.m.sess[s] = make_int2((int)((hw & ~RK_FLAGS) | (fl & RK_FLAGS)), tm);
  r.dirty |= wballot(c.vsid == s);
}
template <int NJ, uint32_t F>
__device__ __forceinline__ void sess_write_flag(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t fl) {
  if (c.lane == 0) c.m.sess[s].x = (int)fl;
  r.dirty |= wballot(c.vsid == s);
}

// ---- timers beyond the 64 sorted ones stay with their session -------------------------------------
// Such a session carries RK_OVF. Its timer is implied by its record: a queued session retries at
// submit time + retries * interval (the duration of its cell waits in a per-replay array in device
// memory), a placed session that is ending ends at its busy-until time. A lower bound of the earliest of them
// is tracked; when the registers run empty, refill() moves up to 64 of them in at once.
template <int NJ, uint32_t F>
__device__ __forceinline__ void ovf_push(Ctx<NJ, F> &c, Regs &r, int32_t t, uint32_t k, int32_t d) {
  const uint32_t s = k & 0xFFFFu;
  if constexpr (Ctx<NJ, F>::closed) {
    // the session's one timer waits in its record: a retry is implied by it as ever, the time of a
    // next event replaces the busy-until time (a closed loop never asks for it)
    if (c.lane == 0) {
      atomicOr((unsigned int *)&c.m.sess[s].x, RK_OVF);
      if ((k >> 16) != QK_RETRY) c.m.sess[s].y = t;
    }
  } else {
    if (c.lane == 0) { atomicOr((unsigned int *)&c.m.sess[s].x, RK_OVF); c.ovf_dur[s] = d; }
  }
  r.dirty |= wballot(c.vsid == s);
  if (r.o_n == 0 || t < r.o_min_t || (t == r.o_min_t && k < r.o_min_k)) { r.o_min_t = t; r.o_min_k = k; }
  r.o_n++;
}

// Registers empty: all timers that are due within a window after the earliest one move
// from the session records into the registers at once, at most 64 (whole instants, so everything
// taken is earlier than everything left behind whatever the kinds; the window adapts to fill 32 to
// 56 registers; more than 64 timers at one instant: the single earliest), and what firing them will
// need is gathered one lane per timer. The same scheme as in the any-size kernel. The kind of a timer
// that is no retry: the deferred end of a busy session (open loop), the session's next event (closed loop).
template <int NJ, uint32_t F>
__device__ __forceinline__ void refill(Ctx<NJ, F> &c, Regs &r) {
  constexpr uint32_t kOther = Ctx<NJ, F>::closed ? QK_NEXT : QK_END;
  wave_sync();
  int cnt;
  int32_t left;                                  // earliest time left behind
  int32_t win = r.cl_win;
  for (;;) {
    const int64_t lim = (int64_t)r.o_min_t + win;
    const int32_t T = lim < NEVER - 1 ? (int32_t)lim : NEVER - 1;
    cnt = 0;
    int32_t mn = NEVER;
    for (int s0 = 0; s0 < c.n_sess; s0 += WAVE) {
      const int s = s0 + c.lane;
      int32_t d = NEVER;
      if (s < c.n_sess) {
        const int2 rec = c.m.sess[s];
        const uint32_t fl = (uint32_t)rec.x;
        if (fl & RK_OVF) d = (fl & 7u) == SS_QUEUED ? rec.y + (int32_t)((fl >> 8) & 15u) * c.p.retry_iv : rec.y;
      }
      const bool hit = d <= T;
      const uint64_t b = wballot(hit);
      if (b != 0) {
        const int pos = cnt + lane_rank(b);
        if (hit && pos < WAVE) c.m.stage[pos] = s;
        cnt += __builtin_popcountll(b);
      }
      mn = hit ? mn : (d < mn ? d : mn);
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
        const int2 rec = c.m.sess[s];
        const uint32_t fl = (uint32_t)rec.x;
        if (fl & RK_OVF) {
          const bool retry = (fl & 7u) == SS_QUEUED;
          const int32_t d = retry ? rec.y + (int32_t)((fl >> 8) & 15u) * c.p.retry_iv : rec.y;
          if (d == T) best = umin(best, ((retry ? QK_RETRY : kOther) << 16) | (uint32_t)s);
        }
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
    const int2 rec = c.m.sess[s];
    const uint32_t fl = (uint32_t)rec.x;
    const bool retry = (fl & 7u) == SS_QUEUED;
    t = retry ? rec.y + (int32_t)((fl >> 8) & 15u) * c.p.retry_iv : rec.y;
    key = ((retry ? QK_RETRY : kOther) << 16) | (uint32_t)s;
    c.m.sess[s].x = (int)(fl & ~RK_OVF);
  }
  // the cursors / durations were written by lane 0 when the timers were scheduled: the fence makes this
  // wave's own stores visible to its other lanes
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  int32_t x = 0, nx = -1, nth = 0;
  if constexpr (Ctx<NJ, F>::closed) {
    if (take) {
      e = c.cl_cur[key & 0xFFFFu];
      const int2 ch = c.cl_chain[e];
      x = c.cl_dur[e] | (int32_t)(((uint32_t)c.cl_sk[e] >> 24) << 28) | CLX_LOADED;
      nx = ch.x; nth = ch.y;
    }
  } else {
    if (take && (key >> 16) == QK_RETRY) e = c.ovf_dur[key & 0xFFFFu];    // qd carries the queued cell's duration
    // the records taken have lost their mark: lanes of the tile that prefetched one read it again. Such a
    // session was queued or ending when the tile was loaded (or its lanes are stale already)
    r.dirty |= r.slow_lanes;
  }
  int rank = 0;
  for (int j = 0; j < cnt; j++) {
    const int32_t tj = lane_get(t, j);
    const uint32_t kj = (uint32_t)lane_get((int)key, j);
    rank += (tj < t || (tj == t && kj < key)) ? 1 : 0;
  }
  const int dst = take ? rank : c.lane;          // a permutation: the timers taken in order, the rest where they are
  c.qt = __builtin_amdgcn_ds_permute(dst << 2, t);
  c.qk = (uint32_t)__builtin_amdgcn_ds_permute(dst << 2, (int)key);
  c.qd = __builtin_amdgcn_ds_permute(dst << 2, e);
  if constexpr (Ctx<NJ, F>::closed) {
    c.qx = __builtin_amdgcn_ds_permute(dst << 2, x);
    c.qnx = __builtin_amdgcn_ds_permute(dst << 2, nx);
    c.qnth = __builtin_amdgcn_ds_permute(dst << 2, nth);
  }
  r.q_n = cnt;
  r.o_n -= cnt;
  r.o_min_t = r.o_n > 0 ? left : NEVER;
  r.o_min_k = 0;                                 // a lower bound: pushes for that very instant wait in the records
}

// ---- hosts ----------------------------------------------------------------------------------------
// committed GPUs of host = lane at time `now`: byte (lane & 7) of the ballot of register (lane >> 3)
template <int NJ, uint32_t F>
__device__ __forceinline__ int committed(const Ctx<NJ, F> &c, int32_t now) {
  const int sh = 8 * (c.lane & 7), grp = c.lane >> 3;
  uint32_t bits = 0;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const uint64_t busy = wballot(c.fin[j] > now);
    const uint32_t mine = (uint32_t)(busy >> sh);
    bits = grp == j ? mine : bits;
  }
  return __builtin_popcount(bits & 0xFFu);
}

// bind g free GPUs of host h until `finish`
template <int NJ, uint32_t F>
__device__ __forceinline__ void bind_gpus(Ctx<NJ, F> &c, int h, int g, int32_t now, int32_t finish) {
  const int j = h >> 3, hl = h & 7;
  const bool mine = (c.lane >> 3) == hl && (c.lane & 7) < c.p.G;
#pragma unroll
  for (int jj = 0; jj < NJ; jj++) {
    if (jj == j) {
      bool fr = mine && c.fin[jj] <= now;
      int rank = lane_rank(wballot(fr));
      if (fr && rank < g) c.fin[jj] = finish;
    }
  }
}

template <int NJ, uint32_t F>
__device__ __forceinline__ int boot_host(Ctx<NJ, F> &c, Regs &r, int32_t now, uint32_t hs_new) {
  uint64_t off = wballot(c.lane < c.p.Hmax && c.hr == NEVER);
  int h = (int)__builtin_ctzll(off);                 // the caller has checked that one exists
  int32_t ra = now + c.p.boot;
  if (c.lane == h) { c.hr = ra; c.hs = hs_new; }
  if (c.flags() & NBOS_F_WARM_POOL) {         // its pre-warmed containers are there once it is up
    if (c.lane < 4) c.m.warm[4 * h + c.lane] = ra + c.p.prewarm;
  }
  c.fu = c.fu < ra ? c.fu : ra;               // a new host may have idle GPUs from then on
  c32_add(c.m, c.lane, CS_NON, 1u);
  c64_add(c.m, c.lane, CL_PROV, -(int64_t)c.p.G * now);
  c32_add(c.m, c.lane, CS_SO, 1u);
  r.lazy_max = r.lazy_max > ra ? r.lazy_max : ra;
  return h;
}

// Earliest time at which some host that is on could have g idle GPUs if nothing new were committed:
// min over hosts of max(ready_at, g-th smallest busy-until time of the host's GPUs). Later commits
// only push it back, so no election or migration for a request of g GPUs can succeed before it
// (as long as no host is added). Each lane counts, inside its host's group of 8 lanes, the GPUs that
// are free no later than its own GPU (DPP quad rotations of the value and of its half-row mirror
// reach all 8 lanes of the group).
template <int NJ, uint32_t F>
__device__ __forceinline__ int32_t earliest_idle(const Ctx<NJ, F> &c, int g) {
  const bool used = (c.lane & 7) < c.p.G;
  int32_t best = NEVER;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const int32_t f = used ? c.fin[j] : NEVER;
    const int32_t mir = __builtin_amdgcn_update_dpp(f, f, 0x141, 0xF, 0xF, false);   // row_half_mirror
    int cnt = 1;
    cnt += __builtin_amdgcn_update_dpp(f, f, 0x39, 0xF, 0xF, false) <= f ? 1 : 0;      // quad_perm [1,2,3,0]
    cnt += __builtin_amdgcn_update_dpp(f, f, 0x4E, 0xF, 0xF, false) <= f ? 1 : 0;      // quad_perm [2,3,0,1]
    cnt += __builtin_amdgcn_update_dpp(f, f, 0x93, 0xF, 0xF, false) <= f ? 1 : 0;      // quad_perm [3,0,1,2]
    cnt += mir <= f ? 1 : 0;
    cnt += __builtin_amdgcn_update_dpp(mir, mir, 0x39, 0xF, 0xF, false) <= f ? 1 : 0;
    cnt += __builtin_amdgcn_update_dpp(mir, mir, 0x4E, 0xF, 0xF, false) <= f ? 1 : 0;
    cnt += __builtin_amdgcn_update_dpp(mir, mir, 0x93, 0xF, 0xF, false) <= f ? 1 : 0;
    const int32_t ra = __builtin_amdgcn_ds_bpermute((8 * j + (c.lane >> 3)) << 2, c.hr);  // ready_at of host 8j+hl
    int32_t y = cnt >= g ? f : NEVER;
    y = y > ra ? y : ra;
    best = best < y ? best : y;
  }
  return (int32_t)wave_min((uint32_t)best);
}

// ---- closed loop: the session's next event is due one think time after `base` --------------------
// r.cl_nx / r.cl_nth: the event after the one being handled and the think time before it. The timer
// carries the event's index; the cursor keeps it for the time the timer waits outside the registers.
template <int NJ, uint32_t F>
__device__ __forceinline__ void cl_schedule(Ctx<NJ, F> &c, Regs &r, uint32_t s, int32_t base) {
  const int32_t e = r.cl_nx;
  if (e < 0) return;
  const int64_t t = (int64_t)base + r.cl_nth;
  if (t >= 0x7FFFFFFFLL) { r.status = NBOS_E_RANGE; return; }
  if (c.lane == 0) c.cl_cur[s] = e;
  timer_push(c, r, (int32_t)t, QK_NEXT, s, e);
}

// ---- SESSION_START: Sections 3.2.1, 3.4.1, 3.4.2 -----------------------------------------------
template <int NJ, uint32_t F>
__device__ __forceinline__ void session_start(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t fl, int32_t now) {
  if ((fl & 7u) != SS_UNPLACED) return;
  const int g = (int)((fl >> 3) & 7u) + 1;
  const int C = committed(c, now);
  const int S = (int)(c.hs & 0xFFFFu);
  const int32_t room = cap_room(c, g);
  uint32_t key = (c.hr <= now && S <= room) ? (((uint32_t)C << 22) | ((uint32_t)S << 10) | (uint32_t)c.lane)
                                            : 0xFFFFFFFFu;
  int pick0 = -1, pick1 = -1, pick2 = -1, k = 0;
  uint32_t m0 = wave_min(key);
  if (m0 != 0xFFFFFFFFu) {
    pick0 = (int)(m0 & 1023u); k = 1;
    key = c.lane == pick0 ? 0xFFFFFFFFu : key;
    uint32_t m1 = wave_min(key);
    if (m1 != 0xFFFFFFFFu) {
      pick1 = (int)(m1 & 1023u); k = 2;
      key = c.lane == pick1 ? 0xFFFFFFFFu : key;
      uint32_t m2 = wave_min(key);
      if (m2 != 0xFFFFFFFFu) { pick2 = (int)(m2 & 1023u); k = 3; }
    }
  }
  const int missing = 3 - k;
  if (missing > 0) {
    wave_sync();
    int n_on = (int)uni(c.m.c32[CS_NON]);
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
      if (c.lane == h) c.hs += add;
      decide(c, r, now, NBOS_D_PLACE, s, (uint32_t)i, (uint32_t)h);
    } else {
      h = boot_host(c, r, now, add);
      decide(c, r, now, NBOS_D_PLACE_NEW, s, (uint32_t)i, (uint32_t)h);
    }
    hw |= (uint32_t)h << (12 + 6 * i);
  }
  if (missing > 0) {
    wave_sync();
    c32_max(c.m, c.lane, CS_PEAK, uni(c.m.c32[CS_NON]));
  }
  sess_write(c, r, s, hw, 0, (fl & ~7u) | SS_PLACED);
  c32_add(c.m, c.lane, CS_PLACED, 1u);
  c32_add(c.m, c.lane, CS_SUMS, (uint32_t)(3 * g));
  c32_add(c.m, c.lane, CS_OPENG, (uint32_t)g);
  c64_add(c.m, c.lane, CL_SUB, -(int64_t)(3 * g) * now);
  c64_add(c.m, c.lane, CL_RESV, -(int64_t)g * now);
  c32_add(c.m, c.lane, CS_NREP, 3u);
  c64_add(c.m, c.lane, CL_REPL, -(int64_t)3 * now);
  if constexpr (Ctx<NJ, F>::closed) cl_schedule(c, r, s, now);
}

// the replicas of session s give their subscriptions back at time `now`
template <int NJ, uint32_t F>
__device__ __forceinline__ void end_session(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int32_t now) {
  const int g = (int)((fl >> 3) & 7u) + 1;
  const uint32_t sub = (uint32_t)g | (1u << 16);
  const int h0 = (int)slot_host(hw, 0), h1 = (int)slot_host(hw, 1), h2 = (int)slot_host(hw, 2);
  if (c.lane == h0 || c.lane == h1 || c.lane == h2) c.hs -= sub;
  sess_write_flag(c, r, s, (fl & ~(7u | SF_ENDING)) | SS_ENDED);
  c32_add(c.m, c.lane, CS_SUMS, (uint32_t)(-3 * g));
  c64_add(c.m, c.lane, CL_SUB, (int64_t)(3 * g) * now);
  c32_add(c.m, c.lane, CS_NREP, (uint32_t)-3);
  c64_add(c.m, c.lane, CL_REPL, (int64_t)3 * now);
}

// ---- a cell starts on (slot, host): Section 3.3 and the metrics of sections "Resource Usage & Efficiency", "Interactivity" and "Task Completion Time" ---------
template <int NJ, uint32_t F>
__device__ __forceinline__ void start_cell(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int slot, int host,
                                           int32_t now, int32_t start, int32_t t_submit, int32_t dur,
                                           uint32_t outcome) {
  const int g = (int)((fl >> 3) & 7u) + 1;
  if constexpr (Ctx<NJ, F>::closed) {         // the lag of a closed loop is not bounded in advance
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
  hw = (hw & ~(63u << (12 + 6 * slot))) | ((uint32_t)host << (12 + 6 * slot));
  // the record's word: hosts and last executor from hw, state back to "placed", retry count cleared
  const uint32_t nw = (hw & ~RK_FLAGS) | (((fl & ~(7u | (15u << 8))) | SS_PLACED) & RK_FLAGS);
  if (__builtin_expect(delay == 0, 1)) {
    r.h0++;                                     // histogram bin 0 lives in a register
    if (c.lane == 0) c.m.sess[s] = make_int2((int)nw, finish);
  } else {
    int b = 32 - __builtin_clz((uint32_t)delay);
    b = b > 31 ? 31 : b;
    if (c.lane == 0) {
      c.m.sess[s] = make_int2((int)nw, finish);
      atomicAdd(&c.m.hist[b], 1u);
      atomicAdd(&c.m.c64[CL_SUMDELAY], (unsigned long long)delay);
      atomicMax(&c.m.c32[CS_MAXDELAY], (uint32_t)delay);
      atomicAdd(&c.m.c64[CL_GWAIT], (unsigned long long)((int64_t)g * (start - now)));
    }
  }
  r.dirty |= wballot(c.vsid == s);
  r.lazy_max = r.lazy_max > finish ? r.lazy_max : finish;
  decide(c, r, now, outcome, s, (uint32_t)slot, (uint32_t)host);
  if (__builtin_expect((fl & SF_ENDING) != 0, 0)) timer_push(c, r, finish, QK_END, s, 0);
  if constexpr (Ctx<NJ, F>::closed) cl_schedule(c, r, s, finish);
}

// ---- executor election, Section 3.2.2 ----------------------------------------------------------------
// key: per lane = host, (committed GPUs << 6) | host where the host is ready and has the GPUs idle, else all
// ones. Among the session's three hosts: fewest committed GPUs, then lowest host index, i.e. the smallest
// of their keys. Returns that key (host in the low 6 bits), or all ones when every replica yields.
template <int NJ, uint32_t F>
__device__ __forceinline__ uint32_t elect(const Ctx<NJ, F> &c, uint32_t hw, uint32_t key) {
  const uint32_t k0 = (uint32_t)lane_get((int)key, (int)slot_host(hw, 0)), k1 = (uint32_t)lane_get((int)key, (int)slot_host(hw, 1)),
                 k2 = (uint32_t)lane_get((int)key, (int)slot_host(hw, 2));
  uint32_t kb = umin(k0, umin(k1, k2));
  if (c.flags() & NBOS_F_STICKY_EXECUTOR) {
    // variant: the replica that ran the previous cell leads again if its host can bind
    const uint32_t last = hw >> 30;
    const uint32_t kp = last == 1u ? k0 : (last == 2u ? k1 : (last == 3u ? k2 : 0xFFFFFFFFu));
    if (kp != 0xFFFFFFFFu) kb = kp;
  }
  return kb;
}

// A cell of an idle placed session starts by election at the instant it is submitted (open loop): what
// start_cell does for a delay of 0, with nothing of the other cases in it.
template <int NJ, uint32_t F>
__device__ __forceinline__ void start_at_once(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t hw, int slot, int host,
                                              int32_t now, int32_t dur) {
  const int g = (int)((hw >> 3) & 7u) + 1;
  const int32_t finish = now + dur;
  r.c_started++;
  r.c_imm++;
  r.h0++;
  r.sum_dur += dur;
  r.g_exec += (int64_t)g * dur;
  if ((hw >> 30) == (uint32_t)slot + 1u) r.reused++;
  // the record's word: hosts as they are, this slot the last executor; state "placed", retry count 0 already
  const uint32_t nw = (hw & 0x3FFFFFFFu) | ((uint32_t)(slot + 1) << 30);
  if (c.lane == 0) c.m.sess[s] = make_int2((int)nw, finish);
  r.dirty |= wballot(c.vsid == s);
  r.lazy_max = r.lazy_max > finish ? r.lazy_max : finish;
  decide(c, r, now, NBOS_D_START, s, (uint32_t)slot, (uint32_t)host);
}

// ---- one attempt to run the pending cell of session s at time `now` -----------------------------
template <int NJ, uint32_t F>
__device__ __forceinline__ void attempt(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int32_t now,
                                        int32_t t_submit, int32_t dur) {
  const int g = (int)((fl >> 3) & 7u) + 1;
  const uint32_t h0 = slot_host(hw, 0), h1 = slot_host(hw, 1), h2 = slot_host(hw, 2);
  // Known in advance that no host has g idle GPUs yet? Then neither election nor migration can work.
  const bool hopeless = now < lane_get(c.fu, g - 1);
  int C = 0;
  uint64_t idle_ok = 0;
  uint32_t kb = 0xFFFFFFFFu;
  if (!hopeless) {
    C = committed(c, now);
    const bool can = c.hr <= now && C + g <= c.p.G;       // a ready host with g idle GPUs
    idle_ok = wballot(can);
    // (a) election, Section 3.2.2: among the session's hosts that can bind, fewest committed GPUs, then
    // lowest host index: the smallest of the three hosts' keys
    kb = elect(c, hw, can ? (((uint32_t)C << 6) | (uint32_t)c.lane) : 0xFFFFFFFFu);
  }
  if (kb != 0xFFFFFFFFu) {
    const int hl = (int)(kb & 63u);
    const int lead = (uint32_t)hl == h0 ? 0 : ((uint32_t)hl == h1 ? 1 : 2);
    bind_gpus(c, hl, g, now, now + dur);
    if (now == t_submit) r.c_imm++;
    start_cell(c, r, s, hw, fl, lead, hl, now, now, t_submit, dur, NBOS_D_START);
    return;
  }
  // No host at all with g idle GPUs: work out when the first one could have them, once, for every
  // later attempt with a request of g or more (commits only push that time back; a booted host
  // lowers it again, see boot_host).
  if (!hopeless && idle_ok == 0) {
    const int32_t bound = earliest_idle(c, g);
    if (c.lane >= g - 1 && c.fu < bound) c.fu = bound;
  }
  // (b), (c): a target exists? Only then is the replica to move worked out: the one on the fullest
  // ready host (ties: lowest host); replicas on booting hosts only if all three are.
  const int S = (int)(c.hs & 0xFFFFu);
  uint64_t target = 0;
  if ((c.flags() & NBOS_F_MIGRATE) && idle_ok != 0) target = idle_ok & wballot(S <= cap_room(c, g));
  bool grow = false;
  if (target == 0 && (c.flags() & NBOS_F_SCALE_OUT)) {
    wave_sync();
    grow = (int)uni(c.m.c32[CS_NON]) < c.p.Hmax;
  }
  if (target != 0 || grow) {
    if (hopeless) C = committed(c, now);
    const uint64_t rdy = wballot(c.hr <= now);
    const int C0 = lane_get(C, (int)h0), C1 = lane_get(C, (int)h1), C2 = lane_get(C, (int)h2);
    const int ok0 = (int)((rdy >> h0) & 1u), ok1 = (int)((rdy >> h1) & 1u), ok2 = (int)((rdy >> h2) & 1u);
    const int any_ready = ok0 | ok1 | ok2;
    const uint32_t v0 = (!any_ready || ok0) ? (((uint32_t)(8 - C0) << 12) | (h0 << 2) | 0u) : 0xFFFFFFFFu;
    const uint32_t v1 = (!any_ready || ok1) ? (((uint32_t)(8 - C1) << 12) | (h1 << 2) | 1u) : 0xFFFFFFFFu;
    const uint32_t v2 = (!any_ready || ok2) ? (((uint32_t)(8 - C2) << 12) | (h2 << 2) | 2u) : 0xFFFFFFFFu;
    const uint32_t vb = umin(v0, umin(v1, v2));
    const int victim = (int)(vb & 3u), hv = (int)((vb >> 2) & 1023u);
    const uint32_t moved = (uint32_t)g | (1u << 16);
    if (target != 0) {
      // (b) migration, Section 3.2.3: the target binds the GPUs at once. A ready host of this session
      // with g idle GPUs would have won the election, so none of its hosts can show up as a target.
      const uint32_t key = ((target >> c.lane) & 1u) ? (((uint32_t)C << 22) | ((uint32_t)S << 10) | (uint32_t)c.lane)
                                                      : 0xFFFFFFFFu;
      const int dst = (int)(wave_min(key) & 1023u);
      bool warm = false;
      if (c.flags() & NBOS_F_WARM_POOL) {
        // Section 3.2.3: the target's pre-warmed container that has been available longest, if any
        // is available now, shortens the start; its replacement is there one pre-warm time later
        wave_sync();
        const uint32_t av = c.lane < c.p.warm_n ? (uint32_t)c.m.warm[4 * dst + c.lane] : 0xFFFFFFFFu;
        const uint32_t first = wave_min(av);
        if ((int32_t)first <= now) {
          const int w = (int)__builtin_ctzll(wballot(av == first));
          if (c.lane == w) c.m.warm[4 * dst + w] = now + c.p.prewarm;
          c32_add(c.m, c.lane, CS_MIGRWARM, 1u);
          warm = true;
        }
      }
      if (c.lane == hv) c.hs -= moved;
      if (c.lane == dst) c.hs += moved;
      c32_add(c.m, c.lane, CS_MIGR, 1u);
      if (warm) {
        const int32_t start = now + c.p.warm_migr;
        bind_gpus(c, dst, g, now, start + dur);
        start_cell(c, r, s, hw, fl, victim, dst, now, start, t_submit, dur, NBOS_D_MIGRATE_WARM);
      } else {
        const int32_t start = now + c.p.migr;
        bind_gpus(c, dst, g, now, start + dur);
        start_cell(c, r, s, hw, fl, victim, dst, now, start, t_submit, dur, NBOS_D_MIGRATE);
      }
    } else {
      // (c) a new host for the cell, Section 3.4.2: reserved and bound before it is up
      const int32_t start = now + c.p.boot + c.p.migr;
      if (c.lane == hv) c.hs -= moved;
      const int h = boot_host(c, r, now, moved);
      wave_sync();
      c32_max(c.m, c.lane, CS_PEAK, uni(c.m.c32[CS_NON]));
      bind_gpus(c, h, g, now, start + dur);
      c32_add(c.m, c.lane, CS_MIGR, 1u);
      start_cell(c, r, s, hw, fl, victim, h, now, start, t_submit, dur, NBOS_D_SCALE_CELL);
    }
    return;
  }
  // (d) queue and retry periodically, then give up, Section 3.2.3
  int retries = (int)((fl >> 8) & 15u);
  if (retries < c.p.max_retries) {
    const bool first = retries == 0;             // an arrival comes in with the count at 0, a retry never
    retries++;
    // A retry that is bound to fail only bumps the retry count: skip straight to the first retry
    // that could succeed (or to the last one, which aborts). Valid while no host can be added:
    // not with the periodic auto-scaler, and not when hosts can be both released and provisioned.
    if (!(c.flags() & NBOS_F_AUTOSCALE) &&
        (c.flags() & (NBOS_F_SCALE_IN | NBOS_F_SCALE_OUT)) != (NBOS_F_SCALE_IN | NBOS_F_SCALE_OUT)) {
      const int32_t bound = lane_get(c.fu, g - 1);
      while (retries < c.p.max_retries && t_submit + retries * c.p.retry_iv < bound) retries++;
    }
    const uint32_t nfl = (fl & ~(7u | (15u << 8))) | SS_QUEUED | ((uint32_t)retries << 8);
    if (first) {                                 // first time in the queue: the submit time goes in
      c32_add(c.m, c.lane, CS_QUEUED, 1u);
      if (c.lane == 0) c.m.sess[s] = make_int2((int)nfl, t_submit);
    } else {
      if (c.lane == 0) c.m.sess[s].x = (int)nfl;
    }
    r.dirty |= wballot(c.vsid == s);
    if constexpr (Ctx<NJ, F>::closed) {
      // every timer carries its event (the cursor still points at the cell under way)
      if ((int64_t)t_submit + (int64_t)retries * c.p.retry_iv >= 0x7FFFFFFFLL) { r.status = NBOS_E_RANGE; return; }
      timer_push(c, r, t_submit + retries * c.p.retry_iv, QK_RETRY, s, r.cl_e, r.cl_x, r.cl_nx, r.cl_nth);
    } else {
      timer_push(c, r, t_submit + retries * c.p.retry_iv, QK_RETRY, s, dur);
    }
    return;
  }
  c32_add(c.m, c.lane, CS_ABORTED, 1u);
  decide(c, r, now, NBOS_D_ABORT, s, 0, 0);
  const uint32_t nfl = (fl & ~(7u | (15u << 8))) | SS_PLACED;
  sess_write(c, r, s, hw, 0, nfl);
  if (fl & SF_ENDING) end_session(c, r, s, hw, nfl, now);
  if constexpr (Ctx<NJ, F>::closed) cl_schedule(c, r, s, now);
}

// ---- runs of retries that fail again ---------------------------------------------------------------
// On a saturated cluster most timers are retries of queued cells (Section 3.2.3) that fail once more:
// no replica's host can bind the GPUs, no migration target, no host to add. Such an attempt changes
// nothing but the session's retry count and its place in the timer queue. This loop takes due
// retries off the head of the sorted registers for as long as they are of that kind (same tests as
// attempt(), same order), re-inserting each with one pass over the registers; the first timer that
// needs anything else is left for the general path. A retry that fails with no retries left gives its
// cell up right here. t_limit = time of the next arrival (timers due
// at or before it run first), tick_t = next auto-scaler period (a timer due at the same time runs
// before it). Returns the time of the last retry handled, or -1. CROWDED: timers are waiting in the session
// records as well (more than 64 pending); a retry that is then no longer earlier than all of those goes to
// wait there too, and the registers are refilled when they run empty. Two instances, so that the common
// case keeps its shorter loop.
template <bool CROWDED, int NJ, uint32_t F>
__device__ __forceinline__ int32_t failing_retries(Ctx<NJ, F> &c, Regs &r, int32_t t_limit, int32_t tick_t) {
  int32_t last = -1;
  const int32_t due = t_limit < tick_t ? t_limit : tick_t;
  const bool may_skip = !(c.flags() & NBOS_F_AUTOSCALE) &&
                        (c.flags() & (NBOS_F_SCALE_IN | NBOS_F_SCALE_OUT)) != (NBOS_F_SCALE_IN | NBOS_F_SCALE_OUT);
  while (r.q_n > 0 && (CROWDED || r.o_n == 0) && r.q_head_t <= due) {
    const int32_t now = r.q_head_t;
    const uint32_t key = (uint32_t)lane_get((int)c.qk, 0);
    if ((key >> 16) != QK_RETRY) break;
    const uint32_t s = key & 0xFFFFu;
    wave_sync();
    const int2 rec = c.m.sess[s];
    const uint32_t hw = uni((uint32_t)rec.x), fl = hw;
    const int32_t t_submit = uni(rec.y);
    int retries = (int)((fl >> 8) & 15u);
    const bool give_up = retries >= c.p.max_retries;           // no retry left: the cell is aborted
    if (give_up && (fl & SF_ENDING)) break;                    // ... and the session ends: general path
    const int g = (int)((fl >> 3) & 7u) + 1;
    if (now >= lane_get(c.fu, g - 1)) {
      const int C = committed(c, now);
      const bool can = c.hr <= now && C + g <= c.p.G;
      if (elect(c, hw, can ? (uint32_t)c.lane : 0xFFFFFFFFu) != 0xFFFFFFFFu) break;   // the election succeeds
      const uint64_t idle_ok = wballot(can);
      if (idle_ok == 0) {
        const int32_t bound = earliest_idle(c, g);
        if (c.lane >= g - 1 && c.fu < bound) c.fu = bound;
      } else if (c.flags() & NBOS_F_MIGRATE) {
        const int S = (int)(c.hs & 0xFFFFu);
        if (idle_ok & wballot(S <= cap_room(c, g))) break;                        // a migration target
      }
    }
    if (c.flags() & NBOS_F_SCALE_OUT) {
      wave_sync();
      if ((int)uni(c.m.c32[CS_NON]) < c.p.Hmax) break;                            // a host can be added
    }
    last = now;
    if (__builtin_expect(give_up, 0)) {
      // it fails for the last time: the cell is given up, the session is idle again, the timer goes
      c32_add(c.m, c.lane, CS_ABORTED, 1u);
      decide(c, r, now, NBOS_D_ABORT, s, 0, 0);
      if (c.lane == 0) c.m.sess[s] = make_int2((int)((fl & ~(7u | (15u << 8))) | SS_PLACED), 0);
      r.dirty |= wballot(c.vsid == s);
      c.qt = __builtin_amdgcn_update_dpp(c.qt, c.qt, 0x130, 0xF, 0xF, false);                      // wave_shl:1
      c.qd = __builtin_amdgcn_update_dpp(c.qd, c.qd, 0x130, 0xF, 0xF, false);
      c.qk = (uint32_t)__builtin_amdgcn_update_dpp((int)c.qk, (int)c.qk, 0x130, 0xF, 0xF, false);
      r.q_n--;
      if constexpr (CROWDED) { if (r.q_n == 0 && r.o_n > 0) refill(c, r); }
      r.q_head_t = r.q_n > 0 ? lane_get(c.qt, 0) : NEVER;
      continue;
    }
    // it fails again: bump the retry count (skipping retries that are bound to fail as well) ...
    retries++;
    if (may_skip) {
      const int32_t bound = lane_get(c.fu, g - 1);
      while (retries < c.p.max_retries && t_submit + retries * c.p.retry_iv < bound) retries++;
    }
    const uint32_t nfl = (fl & ~(15u << 8)) | ((uint32_t)retries << 8);
    if (c.lane == 0) c.m.sess[s].x = (int)nfl;
    r.dirty |= wballot(c.vsid == s);
    // ... and move the entry from lane 0 to its new place: entries before it shift down one lane
    const int32_t t_new = t_submit + retries * c.p.retry_iv;
    const int32_t st = __builtin_amdgcn_update_dpp(c.qt, c.qt, 0x130, 0xF, 0xF, false);          // wave_shl:1
    const int32_t sd = __builtin_amdgcn_update_dpp(c.qd, c.qd, 0x130, 0xF, 0xF, false);
    const uint32_t sk = (uint32_t)__builtin_amdgcn_update_dpp((int)c.qk, (int)c.qk, 0x130, 0xF, 0xF, false);
    const int32_t d_own = lane_get(c.qd, 0);
    if constexpr (CROWDED) {
      if (r.o_n > 0 && !(t_new < r.o_min_t || (t_new == r.o_min_t && key < r.o_min_k))) {
        // no longer earlier than all that waits in the records: the timer goes there, off the registers
        ovf_push(c, r, t_new, key, d_own);
        c.qt = st; c.qd = sd; c.qk = sk;
        r.q_n--;
        if (r.q_n == 0 && r.o_n > 0) refill(c, r);
        r.q_head_t = r.q_n > 0 ? lane_get(c.qt, 0) : NEVER;
        continue;
      }
    }
    const bool before = c.lane >= 1 && c.lane < r.q_n && (c.qt < t_new || (c.qt == t_new && c.qk < key));
    const int pos = __builtin_popcountll(wballot(before));
    if (c.lane < pos) { c.qt = st; c.qd = sd; c.qk = sk; }
    if (c.lane == pos) { c.qt = t_new; c.qd = d_own; c.qk = key; }
    r.q_head_t = lane_get(c.qt, 0);
  }
  return last;
}

// ---- auto-scaler period (Section 3.4.2) -----------------------------------------------------------
// release the highest-numbered ready host without replicas
template <int NJ, uint32_t F>
__device__ __forceinline__ void release_host(Ctx<NJ, F> &c, Regs &r, int32_t now) {
  const uint64_t e = wballot(c.hr <= now && (c.hs >> 16) == 0);
  const int victim = 63 - (int)__builtin_clzll(e);
  if (c.lane == victim) c.hr = NEVER;
  c32_add(c.m, c.lane, CS_NON, (uint32_t)-1);
  c64_add(c.m, c.lane, CL_PROV, (int64_t)c.p.G * now);
  c32_add(c.m, c.lane, CS_SI, 1u);
  decide(c, r, now, NBOS_D_SCALE_IN, 0, 0, (uint32_t)victim);
}

template <int NJ, uint32_t F>
__device__ __forceinline__ void tick(Ctx<NJ, F> &c, Regs &r, int32_t now) {
  int A = __builtin_popcountll(wballot(c.hr <= now));
  int Z = __builtin_popcountll(wballot(c.hr <= now && (c.hs >> 16) == 0));
  int released = 0;
  if (c.flags() & NBOS_F_AUTOSCALE) {
    // expected capacity f * sum C in whole hosts plus the scaling buffer; hosts being provisioned
    // count as capacity
    uint32_t sum_c = 0;
#pragma unroll
    for (int j = 0; j < NJ; j++) sum_c += (uint32_t)__builtin_popcountll(wballot(c.fin[j] > now));
    const uint32_t per_host = 1000u * (uint32_t)c.p.G;
    const int want = (int)(((uint32_t)c.p.f_milli * sum_c + per_host - 1u) / per_host) + c.p.buffer;
    wave_sync();
    int n_on = (int)uni(c.m.c32[CS_NON]);
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

template <int NJ, uint32_t F>
__device__ __forceinline__ void on_session_end(Ctx<NJ, F> &c, Regs &r, uint32_t s, uint32_t hw, int32_t tm, uint32_t fl,
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

// ---- closed-loop kernel: LDS layout of one replay and its initial state (S0) ---------------------------
// (the open-loop kernel below has both written out in its prologue: sharing them cost it 0.7 %)
__device__ __forceinline__ Lds lds_carve_closed(const KParams &p, unsigned char *q) {
  Lds m;
  m.c64 = (unsigned long long *)q; q += 8 * 8;
  m.c32 = (uint32_t *)q;       q += 16 * 4;
  m.hist = (uint32_t *)q;      q += 32 * 4;
  m.sess = (int2 *)q;          q += (size_t)p.n_cap * 8;     // at a fixed offset: its accesses fold it in
  m.stage = (int32_t *)q;      q += WAVE * 4;
  m.warm = (int32_t *)q;                                     // only there with the pool
  return m;
}

// hosts 0..H0-1 ready at time 0, the rest off (in the caller's registers); sessions unplaced
__device__ __forceinline__ void lds_init_closed(const KParams &p, const Lds &m, int lane, int s_lo, int n_sess) {
  if (lane < 8) m.c64[lane] = 0;
  if (lane < 16) m.c32[lane] = lane == CS_NON || lane == CS_PEAK ? (uint32_t)p.H0 : 0u;
  if (lane < 32) m.hist[lane] = 0;
  if (p.warm_n > 0) {
    for (int i = lane; i < WAVE * 4; i += WAVE) m.warm[i] = 0;     // initial hosts: warm from time 0
  }
  for (int s = lane; s < n_sess; s += WAVE) {
    uint32_t g = p.sess_gpus[s_lo + s];
    m.sess[s] = make_int2((int)(SS_UNPLACED | ((g - 1u) << 3)), 0);
  }
  __syncthreads();
}

// ---- S10: close the integrals at t_end and write the result record ---------------------------------
__device__ __forceinline__ void write_stats(const KParams &p, const Lds &m, const Regs &r, int rep, int lane) {
  __syncthreads();
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
    out->sum_delay_ms = sum_delay; out->sum_tct_ms = r.sum_dur + sum_delay;
    out->gpu_ms_executed = r.g_exec; out->gpu_ms_committed = r.g_exec + g_wait;
    out->gpu_ms_provisioned = (int64_t)m.c64[CL_PROV] + (int64_t)m.c32[CS_NON] * p.G * t_end;
    out->reservation_gpu_ms = (int64_t)m.c64[CL_RESV] + (int64_t)(int32_t)m.c32[CS_OPENG] * t_end;
    out->sub_gpu_ms = (int64_t)m.c64[CL_SUB] + (int64_t)(int32_t)m.c32[CS_SUMS] * t_end;
    out->replica_ms = (int64_t)m.c64[CL_REPL] + (int64_t)(int32_t)m.c32[CS_NREP] * t_end;
    out->digest = r.digest;
  }
}

// At most 128 vector registers (4 waves per SIMD): with 8-byte session records a compute unit then holds
// 16 replays of 1,000 sessions at once.
template <int NJ, uint32_t F>
__global__ void __launch_bounds__(WAVE, 4) nbos_replay_reg_kernel(KParams p) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int rep = launch_slot_replay(p);
  const int lane = threadIdx.x;
  if (rep >= p.n_replays) return;
  // launched without a look at the traces on the host: the validation kernel's verdict comes first
  if (p.trace_err != nullptr && *p.trace_err != 0) { refuse_replay(p, rep, lane, NBOS_E_RANGE); return; }

  const int trace = p.trace_of_replay[rep];
  const int64_t ev_lo = p.ev_offset[trace], ev_hi = p.ev_offset[trace + 1];
  const int s_lo = p.sess_offset[trace];
  const int n_sess = p.sess_offset[trace + 1] - s_lo;
  if (p.trace_err != nullptr && n_sess > p.n_cap) { refuse_replay(p, rep, lane, NBOS_E_LIMIT); return; }

  Lds m;
  unsigned char *q = lds_raw;
  m.c64 = (unsigned long long *)q; q += 8 * 8;
  m.c32 = (uint32_t *)q;       q += 16 * 4;
  m.hist = (uint32_t *)q;      q += 32 * 4;
  m.sess = (int2 *)q;          q += (size_t)p.n_cap * 8;     // at a fixed offset: its accesses fold it in
  m.stage = (int32_t *)q;      q += WAVE * 4;
  m.warm = (int32_t *)q;                                     // only there with the pool

  // S0: hosts 0..H0-1 ready at time 0, the rest off; sessions unplaced
  if (lane < 8) m.c64[lane] = 0;
  if (lane < 16) m.c32[lane] = lane == CS_NON || lane == CS_PEAK ? (uint32_t)p.H0 : 0u;
  if (lane < 32) m.hist[lane] = 0;
  if (p.warm_n > 0) {
    for (int i = lane; i < WAVE * 4; i += WAVE) m.warm[i] = 0;     // initial hosts: warm from time 0
  }
  for (int s = lane; s < n_sess; s += WAVE) {
    uint32_t g = p.sess_gpus[s_lo + s];
    m.sess[s] = make_int2((int)(SS_UNPLACED | ((g - 1u) << 3)), 0);
  }
  __syncthreads();

  const int32_t caplim = p.cap_milli[rep] * p.G * 3;
  Ctx<NJ, F> c{p, m, lane, n_sess, caplim / 1000, p.dlog ? p.dlog + (int64_t)rep * p.dlog_stride : nullptr,
               p.ovf_dur + (int64_t)rep * p.n_cap};
#pragma unroll
  for (int j = 0; j < NJ; j++) c.fin[j] = 0;
  c.hr = lane < p.H0 ? 0 : NEVER;
  c.hs = 0;
  c.qt = NEVER; c.qd = 0; c.qk = 0xFFFFFFFFu;
  c.vsid = 0xFFFFFFFFu;
  c.fu = 0;
  c.dyn = dynamic_limit_matters(p, c.flags(), c.slim);
  Regs r;
  memset(&r, 0, sizeof r);
  r.digest = 0xCBF29CE484222325ULL;
  r.q_head_t = NEVER;
  r.o_min_t = NEVER;
  r.cl_win = 1024;

  const bool ticking = (c.flags() & (NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE)) != 0;
  int32_t tick_t = ticking ? p.scale_iv : NEVER;
  int32_t due_t = tick_t;                   // earliest queued timer or auto-scaler period
  PROF_BEGIN();

  // S1: stream the events, one per lane per tile, next tile in flight
  int64_t base = ev_lo;                     // first event of the tile held in (nt, nd, ns)
  int32_t vt = 0, vd = 0, vs = 0, nt = 0, nd = 0, ns = 0;
  if (base + lane < ev_hi) { nt = p.ev_time[base + lane]; nd = p.ev_dur[base + lane]; ns = p.ev_sk[base + lane]; }

  // Outer loop: one iteration per tile of 64 events plus a last one (`final`) that drains the
  // timers. Inner loop: one iteration per item (queued timer, auto-scaler period, or arrival); it
  // never touches the registers of the tile in flight.
  bool final = false;
  while (r.status == NBOS_OK) {
    int2 rec = make_int2(0, 0);             // prefetched session record of this lane's event
    uint32_t fast = 0;                      // this lane's event is a cell of an idle placed session
    bool base_valid_cell = false;           // this lane's event is a cell
    uint64_t todo = 0;
    if (base < ev_hi) {
      // the prefetched tile becomes current; start loading the one after it
      vt = nt; vd = nd; vs = ns;
      const int64_t cur = base;
      base += WAVE;
      if (base + lane < ev_hi) { nt = p.ev_time[base + lane]; nd = p.ev_dur[base + lane]; ns = p.ev_sk[base + lane]; }
      const bool valid = cur + lane < ev_hi;
      const bool is_last = cur + lane == ev_hi - 1;
      const uint32_t sid = (uint32_t)vs & 0xFFFFFFu;
      const bool is_cell = ((uint32_t)vs >> 24) == NBOS_EV_CELL;
      c.vsid = valid ? sid : 0xFFFFFFFFu;
      wave_sync();
      if (valid) rec = m.sess[sid];
      // Cells of sessions in a final state (rejected / ended) and cells that arrive while the
      // session's running cell lasts beyond them change nothing: count them, skip them. Neither
      // condition can be undone before the event's time. The last event of the trace is never
      // skipped, so timers due before it still run first.
      const uint32_t st = (uint32_t)rec.x & 7u;
      const bool dead = st == SS_REJECTED || st == SS_ENDED;
      const bool running = st == SS_PLACED && rec.y > vt;
      const bool skip = valid && !is_last && (dead || (is_cell && running));
      r.c_total += (uint32_t)__builtin_popcountll(wballot(valid && is_cell));
      r.c_unplaced += (uint32_t)__builtin_popcountll(wballot(skip && is_cell && dead));
      r.c_busy += (uint32_t)__builtin_popcountll(wballot(skip && is_cell && !dead));
      fast = (valid && is_cell && st == SS_PLACED && !running && !((uint32_t)rec.x & SF_ENDING)) ? 1u : 0u;
      base_valid_cell = valid && is_cell;
      todo = wballot(valid && !skip);
      r.dirty = 0;
      if (ev_hi - cur <= WAVE) {
        int32_t tl = lane_get(vt, (int)(ev_hi - cur - 1));
        r.t_end = r.t_end > tl ? r.t_end : tl;
      }
    } else {
      final = true;
    }
    const uint64_t fastmask = wballot(fast != 0);
    PROF(PC_TILE, 1);
    const uint64_t cellmask = wballot(base_valid_cell);
    r.slow_lanes = ~fastmask;
    for (;;) {
      if (__builtin_expect(r.status != NBOS_OK, 0)) break;
      // ---- runs of arrivals that start at once (S4, S5): cells of idle placed sessions (by the prefetched
      // record, or, where that is stale, by the record as it is now), no timer due first, the election won.
      // A loop of its own with nothing else in it; whatever does not fit leaves the arrival to the general
      // path below.
      PROF(PC_LOOP_ROUND, 1);
      [[maybe_unused]] const uint32_t prof_imm0 = r.c_imm;
      while (todo != 0) {
        const int i = (int)__builtin_ctzll(todo);
        if (((cellmask >> i) & 1ull) == 0) break;
        const int32_t t = lane_get(vt, i);
        if (t >= due_t) break;
        uint32_t hw;
        if ((((fastmask & ~r.dirty) >> i) & 1ull) != 0) {
          hw = (uint32_t)lane_get(rec.x, i);
        } else {
          wave_sync();
          const int2 cur = m.sess[(uint32_t)lane_get(vs, i) & 0xFFFFFFu];
          hw = uni((uint32_t)cur.x);
          // idle and placed, nothing pending (the general path copes with everything else)
          if ((hw & (7u | SF_ENDING | RK_OVF | (15u << 8))) != SS_PLACED || uni(cur.y) > t) break;
        }
        const int g = (int)((hw >> 3) & 7u) + 1;
        if (t < lane_get(c.fu, g - 1)) break;                 // no host has g idle GPUs yet
        // election (Section 3.2.2) on the vector side: every host's key (committed GPUs, index), or all
        // ones where it cannot bind; the keys of the session's three hosts are read and compared
        const int C = committed(c, t);
        const uint32_t key = (c.hr <= t && C + g <= c.p.G) ? (((uint32_t)C << 6) | (uint32_t)c.lane) : 0xFFFFFFFFu;
        const uint32_t kb = elect(c, hw, key);
        if (kb == 0xFFFFFFFFu) break;                         // every replica yields
        const int hl = (int)(kb & 63u);
        const int lead = (uint32_t)hl == slot_host(hw, 0) ? 0 : ((uint32_t)hl == slot_host(hw, 1) ? 1 : 2);
        const int32_t dur = lane_get(vd, i);
        bind_gpus(c, hl, g, t, t + dur);
        start_at_once(c, r, (uint32_t)lane_get(vs, i) & 0xFFFFFFu, hw, lead, hl, t, dur);
        todo &= todo - 1;
      }
      PROF(PC_ROUND, r.c_imm - prof_imm0);
      int i = 0;
      int32_t t = NEVER;
      if (todo != 0) { i = (int)__builtin_ctzll(todo); t = lane_get(vt, i); }
      else if (!final) break;
      wave_sync();
      uint32_t a_s, a_hw, a_fl;
      int32_t a_now, a_sub, a_dur;
      [[maybe_unused]] bool is_retry = false;      // (path profile)
      if (__builtin_expect(t < due_t, 1)) {
        // ---- arrival i ----
        const uint64_t bit = 1ull << i;
        todo &= ~bit;
        const uint32_t sk = (uint32_t)lane_get(vs, i);
        const uint32_t s = sk & 0xFFFFFFu;
        if (__builtin_expect((fastmask & ~r.dirty & bit) != 0, 1)) {
          // a cell of an idle placed session whose record nobody touched since the prefetch
          a_s = s; a_hw = (uint32_t)lane_get(rec.x, i);
          a_fl = a_hw;
          a_now = t; a_sub = t; a_dur = lane_get(vd, i);
        } else {
          const uint32_t kind = sk >> 24;
          uint32_t hw, fl;
          int32_t tm;
          if ((r.dirty >> i) & 1u) {
            int2 cur = m.sess[s];
            hw = uni((uint32_t)cur.x); tm = uni(cur.y); fl = hw;
          } else {
            hw = (uint32_t)lane_get(rec.x, i); tm = lane_get(rec.y, i); fl = hw;
          }
          if (kind == NBOS_EV_CELL) {           // S4-S8 (counted in c_total at tile load)
            const uint32_t st = fl & 7u;
            if (st == SS_PLACED && tm <= t) {
              a_s = s; a_hw = hw; a_fl = fl & ~(15u << 8); a_now = t; a_sub = t; a_dur = lane_get(vd, i);
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
        {
          const int32_t last = r.o_n == 0 ? failing_retries<false>(c, r, t, tick_t) : failing_retries<true>(c, r, t, tick_t);
          PROF(PC_QUIET_RETRIES, 1);
          if (last >= 0) {
            r.t_end = r.t_end > last ? r.t_end : last;
            due_t = r.q_head_t < tick_t ? r.q_head_t : tick_t;
            if (t < due_t) continue;
          }
        }
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
        const int32_t now = r.q_head_t;
        const uint32_t key = (uint32_t)lane_get((int)c.qk, 0);
        const int32_t dur = lane_get(c.qd, 0);
        const uint32_t s = key & 0xFFFFu;
        const int2 cur = m.sess[s];           // (asked for before the pop, which does not touch this record)
        timer_pop(c, r);
        r.t_end = r.t_end > now ? r.t_end : now;
        const uint32_t hw = uni((uint32_t)cur.x), fl = hw;
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
      attempt(c, r, a_s, a_hw, a_fl, a_now, a_sub, a_dur);
      PROF_ATTEMPT_END(m, r, is_retry);
      due_t = r.q_head_t < tick_t ? r.q_head_t : tick_t;
    }
    if (final) break;
  }

  write_stats(p, m, r, rep, lane);
  PROF_OUT(rep);
}

// ---- closed loop: runs of retries that fail again (failing_retries() for this kernel) -----------------
// Same tests, same order. The retry's timer either stays in the sorted registers at its new place, or,
// if it is no longer earlier than everything that waits in the session records, goes there. A retry
// with no retries left is left for the general path (giving a cell up schedules the session's next
// event). Returns the time of the last retry handled, or -1.
template <int NJ, uint32_t F>
__device__ __forceinline__ int32_t cl_failing_retries(Ctx<NJ, F> &c, Regs &r, int32_t t_limit) {
  int32_t last = -1;
  const bool may_skip = !(c.flags() & NBOS_F_AUTOSCALE) &&
                        (c.flags() & (NBOS_F_SCALE_IN | NBOS_F_SCALE_OUT)) != (NBOS_F_SCALE_IN | NBOS_F_SCALE_OUT);
  while (r.q_n > 0 && r.q_head_t <= t_limit) {
    const int32_t now = r.q_head_t;
    const uint32_t key = (uint32_t)lane_get((int)c.qk, 0);
    if ((key >> 16) != QK_RETRY) break;
    const uint32_t s = key & 0xFFFFu;
    wave_sync();
    const int2 rec = c.m.sess[s];
    const uint32_t hw = uni((uint32_t)rec.x), fl = hw;
    const int32_t t_submit = uni(rec.y);
    int retries = (int)((fl >> 8) & 15u);
    if (retries >= c.p.max_retries) break;                     // it would be given up: general path
    const int g = (int)((fl >> 3) & 7u) + 1;
    if (now >= lane_get(c.fu, g - 1)) {
      const int C = committed(c, now);
      const bool can = c.hr <= now && C + g <= c.p.G;
      if (elect(c, hw, can ? (uint32_t)c.lane : 0xFFFFFFFFu) != 0xFFFFFFFFu) break;   // the election succeeds
      const uint64_t idle_ok = wballot(can);
      if (idle_ok == 0) {
        const int32_t bound = earliest_idle(c, g);
        if (c.lane >= g - 1 && c.fu < bound) c.fu = bound;
      } else if (c.flags() & NBOS_F_MIGRATE) {
        const int S = (int)(c.hs & 0xFFFFu);
        if (idle_ok & wballot(S <= cap_room(c, g))) break;                        // a migration target
      }
    }
    if (c.flags() & NBOS_F_SCALE_OUT) {
      wave_sync();
      if ((int)uni(c.m.c32[CS_NON]) < c.p.Hmax) break;                            // a host can be added
    }
    // it fails again: bump the retry count (skipping retries that are bound to fail as well)
    retries++;
    if (may_skip) {
      const int32_t bound = lane_get(c.fu, g - 1);
      while (retries < c.p.max_retries && t_submit + retries * c.p.retry_iv < bound) retries++;
    }
    if ((int64_t)t_submit + (int64_t)retries * c.p.retry_iv >= 0x7FFFFFFFLL) break;   // out of range: general path
    last = now;
    const uint32_t nfl = (fl & ~(15u << 8)) | ((uint32_t)retries << 8);
    if (c.lane == 0) c.m.sess[s].x = (int)nfl;
    const int32_t t_new = t_submit + retries * c.p.retry_iv;
    const int32_t st = __builtin_amdgcn_update_dpp(c.qt, c.qt, 0x130, 0xF, 0xF, false);          // wave_shl:1
    const int32_t sd = __builtin_amdgcn_update_dpp(c.qd, c.qd, 0x130, 0xF, 0xF, false);
    const uint32_t sk = (uint32_t)__builtin_amdgcn_update_dpp((int)c.qk, (int)c.qk, 0x130, 0xF, 0xF, false);
    const int32_t sx = __builtin_amdgcn_update_dpp(c.qx, c.qx, 0x130, 0xF, 0xF, false);
    const int32_t sn = __builtin_amdgcn_update_dpp(c.qnx, c.qnx, 0x130, 0xF, 0xF, false);
    const int32_t sh = __builtin_amdgcn_update_dpp(c.qnth, c.qnth, 0x130, 0xF, 0xF, false);
    if (r.o_n > 0 && !(t_new < r.o_min_t || (t_new == r.o_min_t && key < r.o_min_k))) {
      // no longer earlier than all that waits in the records: the timer goes there, off the registers
      ovf_push(c, r, t_new, key, 0);
      c.qt = st; c.qd = sd; c.qk = sk; c.qx = sx; c.qnx = sn; c.qnth = sh;
      r.q_n--;
      if (r.q_n == 0 && r.o_n > 0) refill(c, r);
      r.q_head_t = r.q_n > 0 ? lane_get(c.qt, 0) : NEVER;
    } else {
      // it moves from lane 0 to its new place: the entries before that shift down one lane
      const bool before = c.lane >= 1 && c.lane < r.q_n && (c.qt < t_new || (c.qt == t_new && c.qk < key));
      const int pos = __builtin_popcountll(wballot(before));
      const int32_t d_own = lane_get(c.qd, 0), x_own = lane_get(c.qx, 0), n_own = lane_get(c.qnx, 0), h_own = lane_get(c.qnth, 0);
      if (c.lane < pos) { c.qt = st; c.qd = sd; c.qk = sk; c.qx = sx; c.qnx = sn; c.qnth = sh; }
      if (c.lane == pos) { c.qt = t_new; c.qd = d_own; c.qk = key; c.qx = x_own; c.qnx = n_own; c.qnth = h_own; }
      r.q_head_t = lane_get(c.qt, 0);
    }
  }
  return last;
}

// ---- closed-loop reading of the trace (see the file header and nbos_kernel_closed.hpp) -----------------
// Arrivals from the stream are the first STARTs only (the STARTs that head a chain record); every other
// event is a timer of kind QK_NEXT. Timers whose events were not loaded when they were scheduled load
// them together when the first of them gets to the head.
template <int NJ, uint32_t F>
__global__ void __launch_bounds__(WAVE, 4) nbos_replay_reg_closed_kernel(KParams p) {
  static_assert(Ctx<NJ, F>::closed, "instantiate with a closed-loop flag set");
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int rep = launch_slot_replay(p);
  const int lane = threadIdx.x;
  if (rep >= p.n_replays) return;

  const int trace = p.trace_of_replay[rep];
  const int64_t ev_lo = p.ev_offset[trace], ev_hi = p.ev_offset[trace + 1];
  const int s_lo = p.sess_offset[trace];
  const int n_sess = p.sess_offset[trace + 1] - s_lo;

  const Lds m = lds_carve_closed(p, lds_raw);
  lds_init_closed(p, m, lane, s_lo, n_sess);

  const int32_t caplim = p.cap_milli[rep] * p.G * 3;
  Ctx<NJ, F> c{p, m, lane, n_sess, caplim / 1000, p.dlog ? p.dlog + (int64_t)rep * p.dlog_stride : nullptr, nullptr};
#pragma unroll
  for (int j = 0; j < NJ; j++) c.fin[j] = 0;
  c.hr = lane < p.H0 ? 0 : NEVER;
  c.hs = 0;
  c.qt = NEVER; c.qd = 0; c.qk = 0xFFFFFFFFu;
  c.vsid = 0xFFFFFFFFu;
  c.fu = 0;
  c.dyn = dynamic_limit_matters(p, c.flags(), c.slim);
  c.cl_cur = p.cl_cursor + (int64_t)rep * p.n_cap;
  c.cl_dur = p.ev_dur + ev_lo; c.cl_sk = p.ev_sk + ev_lo; c.cl_chain = p.cl_chain + ev_lo;
  c.qx = 0; c.qnx = -1; c.qnth = 0;
  Regs r;
  memset(&r, 0, sizeof r);
  r.digest = 0xCBF29CE484222325ULL;
  r.q_head_t = NEVER;
  r.o_min_t = NEVER;
  r.cl_win = 1024;

  bool final = false;
  for (int64_t base = ev_lo; r.status == NBOS_OK; base += WAVE) {
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
        {
          const int32_t last = cl_failing_retries(c, r, t);
          if (last >= 0) { r.t_end = r.t_end > last ? r.t_end : last; continue; }
        }
        if (!(lane_get(c.qx, 0) & CLX_LOADED) && ((uint32_t)lane_get((int)c.qk, 0) >> 16) != QK_END) {
          if (c.lane < r.q_n && !(c.qx & CLX_LOADED) && (c.qk >> 16) != QK_END) {
            const int2 ch = c.cl_chain[c.qd];
            c.qx = c.cl_dur[c.qd] | (int32_t)(((uint32_t)c.cl_sk[c.qd] >> 24) << 28) | CLX_LOADED;
            c.qnx = ch.x; c.qnth = ch.y;
          }
        }
        const int32_t now = r.q_head_t;
        const uint32_t key = (uint32_t)lane_get((int)c.qk, 0);
        const int32_t e = lane_get(c.qd, 0);
        const int32_t x = lane_get(c.qx, 0), nx = lane_get(c.qnx, 0), nth = lane_get(c.qnth, 0);
        timer_pop(c, r);
        r.t_end = r.t_end > now ? r.t_end : now;
        const uint32_t s = key & 0xFFFFu, kind = key >> 16;
        wave_sync();
        const int2 cur = m.sess[s];
        const uint32_t hw = uni((uint32_t)cur.x), fl = hw;
        const int32_t tm = uni(cur.y);
        if (kind == QK_END) { end_session(c, r, s, hw, fl, now); continue; }
        r.cl_e = e; r.cl_x = x; r.cl_nx = nx; r.cl_nth = nth;
        const int32_t dur = x & 0x0FFFFFFF;
        if (kind == QK_RETRY) {
          attempt(c, r, s, hw, fl, now, tm, dur);
        } else if ((((uint32_t)x >> 28) & 3u) == NBOS_EV_CELL) {     // the session submits its next cell (S4-S8)
          r.c_total++;
          const uint32_t st = fl & 7u;
          // (a session whose next event is due is idle: its time word may hold that due time)
          if (st == SS_PLACED && !(fl & SF_ENDING)) attempt(c, r, s, hw, fl & ~(15u << 8), now, now, dur);
          else if (st == SS_PLACED || st == SS_QUEUED) r.c_busy++;
          else r.c_unplaced++;
        } else {
          on_session_end(c, r, s, hw, now, fl, now);              // S9: idle, so it ends at once
        }
        continue;
      }
      if (todo == 0) break;                 // draining and no timer is left
      todo &= todo - 1;
      const uint32_t s = (uint32_t)lane_get((int)vs, i) & 0xFFFFFFu;
      const uint32_t fl = uni((uint32_t)m.sess[s].x);
      r.t_end = r.t_end > t ? r.t_end : t;
      r.cl_e = (int32_t)(base - ev_lo) + i; r.cl_nx = lane_get(vnx, i); r.cl_nth = lane_get(vnth, i);
      session_start(c, r, s, fl, t);        // S3, S7; a placed session's first event is scheduled there
    }
    if (final) break;
  }
  write_stats(p, m, r, rep, lane);
}

}  // namespace regk
}  // namespace
