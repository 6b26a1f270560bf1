// nbos_kernel_lds.hpp — replay kernel with host state in LDS: any cluster size up to
// NBOS_MAX_HOSTS (several hosts per lane). Used when hosts_max > 64.
//
// One workgroup (one wave64) per replay. Per-replay state in LDS:
//
//   fin[k][h]     per-GPU "busy until" time of GPU k on host h (k-major so that a scan over hosts
//                 is a conflict-free stride-1 read). A GPU is committed at time t iff fin > t.
//                 Dynamic GPU binding (paper Section 3.3) becomes: write the cell's finish time
//                 into g free GPUs of the host. Completions need no timer: a GPU is released the
//                 moment the clock passes its fin. This is exact because every timer due at or
//                 before an item runs before that item, and a completion only lowers C.
//   ready_at[h]   time the host becomes ready (0 for initial hosts, NEVER while off): hosts that
//                 are being provisioned (Section 3.4.2) turn ready without a timer as well.
//   hsn[h]        subscribed GPUs S (low 16 bits) and replica count (high 16 bits), Section 3.4.1.
//   sessions      3 words each: replica hosts (3 x 10 bits) + last executor slot, a time word
//                 (busy-until while running, submit time while queued), flags.
//   queue         the few timers that do change decisions when they fire: RETRY of a queued cell
//                 (Section 3.2.3) and the END of a session that was busy when its END arrived.
//                 Unsorted array, minimum found by a wave-parallel scan.
//
// Lane = host for every scan over hosts (placement, migration target, scale-out, scale-in):
// feasibility by ballot, choice by a packed-key wave minimum (committed, subscribed, index), so
// ties break to the lowest host index. The election (Section 3.2.2) reads the 3 x 8 GPU words of
// the session's replica hosts with 24 lanes and counts committed GPUs with one ballot.
// The event stream is read with coalesced dword loads, one event per lane, the next tile in flight
// while the current one is consumed straight from registers (v_readlane), so events never touch LDS.
#pragma once
#include "nbos_common.hpp"

namespace {
namespace ldsk {

// Uniform per-replay registers (the compiler keeps them on the scalar unit).
struct Regs {
  uint32_t n_dec, placed, rejected, c_total, c_imm, c_started, c_queued, c_aborted, c_busy, c_unplaced;
  uint32_t reused, migrations, so_hosts, si_hosts, peak;
  int32_t max_delay, t_end, lazy_max;
  int64_t sum_delay, sum_tct, g_exec, g_commit, prov, resv, sub;
  uint64_t digest;
  int32_t n_on, sum_s, open_g;   // hosts not off, cluster subscription, GPUs of open Reservation lifetimes
  int32_t q_n, q_min_t, q_min_i; // queue size, time and index of its minimum
  int32_t status;
};

struct Lds {
  int32_t *fin, *ready_at;
  uint32_t *hsn, *hist;
  uint32_t *s_hosts, *s_flag;
  int32_t *s_time;
  int32_t *q_t, *q_d;
  uint32_t *q_i;
};

struct Ctx {
  const KParams &p;
  Lds m;
  int lane;
  int32_t caplim;          // cap_milli * G * 3
  uint64_t *dlog;
};

__device__ __forceinline__ void decide(Ctx &c, Regs &r, int32_t now, uint32_t outcome, uint32_t s,
                                       uint32_t slot, uint32_t host) {
  uint64_t code = (uint64_t)host | ((uint64_t)slot << 10) | ((uint64_t)outcome << 12) |
                  ((uint64_t)s << 16) | ((uint64_t)(uint32_t)now << 32);
  r.digest = r.digest * 0x100000001B3ULL + code;
  if (c.dlog) {
    if (c.lane == 0 && (int64_t)r.n_dec < c.p.dlog_stride) c.dlog[r.n_dec] = code;
  }
  r.n_dec++;
}

// ---- queue of decision-changing timers ----------------------------------------------------------
__device__ __forceinline__ void queue_rescan(Ctx &c, Regs &r) {
  wave_sync();
  uint32_t bt = 0xFFFFFFFFu, bl = 0xFFFFFFFFu;
  int bi = 0;
  for (int i = c.lane; i < r.q_n; i += WAVE) {
    uint32_t t = (uint32_t)c.m.q_t[i], l = c.m.q_i[i];
    if (t < bt || (t == bt && l < bl)) { bt = t; bl = l; bi = i; }
  }
  uint32_t mt = wave_min(bt);
  uint32_t ml = wave_min(bt == mt ? bl : 0xFFFFFFFFu);
  uint64_t who = wballot(bt == mt && bl == ml);
  int src = (int)__builtin_ctzll(who | (1ull << 63));
  r.q_min_i = lane_get(bi, src);
  r.q_min_t = r.q_n > 0 ? (int32_t)mt : NEVER;
}

__device__ __forceinline__ void queue_push(Ctx &c, Regs &r, int32_t t, uint32_t kind, uint32_t id, int32_t dur) {
  wave_sync();
  if (r.q_n >= c.p.q_cap) { r.status = NBOS_E_LIMIT; return; }
  uint32_t key = (kind << 16) | id;
  if (c.lane == 0) { c.m.q_t[r.q_n] = t; c.m.q_i[r.q_n] = key; c.m.q_d[r.q_n] = dur; }
  bool better = r.q_n == 0 || t < r.q_min_t;
  if (!better && t == r.q_min_t) better = key < uni(c.m.q_i[r.q_min_i]);
  if (better) { r.q_min_t = t; r.q_min_i = r.q_n; }
  r.q_n++;
}

// ---- host helpers -------------------------------------------------------------------------------
// committed GPUs of host h at time `now` (one lane per host)
__device__ __forceinline__ int committed(const Ctx &c, int h, int32_t now) {
  int n = 0;
#pragma unroll
  for (int k = 0; k < NGPU; k++)
    if (k < c.p.G) n += c.m.fin[k * c.p.HP + h] > now ? 1 : 0;
  return n;
}

// bind g free GPUs of host h until `finish` (lanes 0..G-1 each look at one GPU)
__device__ __forceinline__ void bind_gpus(Ctx &c, int h, int g, int32_t now, int32_t finish) {
  wave_sync();
  bool mine = c.lane < c.p.G;
  int32_t f = mine ? c.m.fin[c.lane * c.p.HP + h] : NEVER;
  bool fr = mine && f <= now;
  int rank = lane_rank(wballot(fr));
  if (fr && rank < g) c.m.fin[c.lane * c.p.HP + h] = finish;
}

// lowest host index that is off, or -1
__device__ __forceinline__ int find_off_host(const Ctx &c) {
  wave_sync();
  for (int base = 0; base < c.p.HP; base += WAVE) {
    int h = base + c.lane;
    uint64_t off = wballot(h < c.p.Hmax && c.m.ready_at[h] == NEVER);
    if (off) return base + (int)__builtin_ctzll(off);
  }
  return -1;
}

__device__ __forceinline__ void boot_host(Ctx &c, Regs &r, int h, int32_t now) {
  int32_t ra = now + c.p.boot;
  if (c.lane == 0) c.m.ready_at[h] = ra;
  r.n_on++;
  r.peak = r.peak > (uint32_t)r.n_on ? r.peak : (uint32_t)r.n_on;
  r.prov -= (int64_t)c.p.G * now;
  r.lazy_max = r.lazy_max > ra ? r.lazy_max : ra;
}

// Best host for one more replica with request g: ready, under the cap, optionally with g idle GPUs
// now; smallest (committed, subscribed, index). Hosts ex0 / ex1 are skipped. Returns the packed key
// (host in the low 10 bits) or 0xFFFFFFFF.
__device__ __forceinline__ uint32_t best_host(const Ctx &c, int32_t now, int g, bool need_idle, int ex0, int ex1) {
  wave_sync();
  uint32_t best = 0xFFFFFFFFu;
  for (int h = c.lane; h < c.p.HP; h += WAVE) {
    int32_t ra = c.m.ready_at[h];
    int S = (int)(c.m.hsn[h] & 0xFFFFu);
    int C = committed(c, h, now);
    bool ok = ra <= now && (S + g) * 1000 <= c.caplim && h != ex0 && h != ex1;
    if (need_idle) ok = ok && (c.p.G - C >= g);
    uint32_t key = ((uint32_t)C << 22) | ((uint32_t)S << 10) | (uint32_t)h;
    if (ok) best = umin(best, key);
  }
  return wave_min(best);
}

// ---- SESSION_START: Sections 3.2.1, 3.4.1, 3.4.2 -----------------------------------------------
__device__ __forceinline__ void session_start(Ctx &c, Regs &r, uint32_t s, int32_t now) {
  wave_sync();
  uint32_t fl = uni(c.m.s_flag[s]);
  if ((fl & 7u) != SS_UNPLACED) return;
  int g = (int)((fl >> 3) & 7u) + 1;
  int pick[3] = {-1, -1, -1};
  int k = 0;
  for (int i = 0; i < 3; i++) {
    uint32_t key = best_host(c, now, g, false, pick[0], pick[1]);
    if (key == 0xFFFFFFFFu) break;
    pick[i] = (int)(key & 1023u);
    k++;
  }
  int missing = 3 - k;
  if (missing > 0 && !((c.p.flags & NBOS_F_SCALE_OUT) && r.n_on + missing <= c.p.Hmax)) {
    if (c.lane == 0) c.m.s_flag[s] = (fl & ~7u) | SS_REJECTED;
    r.rejected++;
    decide(c, r, now, NBOS_D_REJECT, s, 0, 0);
    return;
  }
  uint32_t hw = 0;
  uint32_t add = (uint32_t)g | (1u << 16);
  for (int i = 0; i < 3; i++) {
    int h;
    if (i < k) {
      h = pick[i];
      if (c.lane == 0) c.m.hsn[h] += add;
      decide(c, r, now, NBOS_D_PLACE, s, (uint32_t)i, (uint32_t)h);
    } else {
      h = find_off_host(c);
      boot_host(c, r, h, now);
      if (c.lane == 0) c.m.hsn[h] = add;
      r.so_hosts++;
      decide(c, r, now, NBOS_D_PLACE_NEW, s, (uint32_t)i, (uint32_t)h);
    }
    hw |= (uint32_t)h << (10 * i);
  }
  if (c.lane == 0) {
    c.m.s_hosts[s] = hw;                     // last executor: none (bits 30..31 = 0)
    c.m.s_flag[s] = (fl & ~7u) | SS_PLACED;
    c.m.s_time[s] = 0;
  }
  r.placed++;
  r.sum_s += 3 * g;
  r.open_g += g;
  r.sub -= (int64_t)(3 * g) * now;
  r.resv -= (int64_t)g * now;
}

// the replicas of session s give their subscriptions back at time `now`
__device__ __forceinline__ void end_session(Ctx &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int32_t now) {
  int g = (int)((fl >> 3) & 7u) + 1;
  uint32_t sub = (uint32_t)g | (1u << 16);
  if (c.lane < 3) {
    int h = (int)((hw >> (10 * c.lane)) & 1023u);
    c.m.hsn[h] -= sub;                        // three distinct hosts, one lane each
  }
  if (c.lane == 0) c.m.s_flag[s] = (fl & ~(7u | SF_ENDING)) | SS_ENDED;
  r.sum_s -= 3 * g;
  r.sub += (int64_t)(3 * g) * now;
}

// ---- a cell starts on (slot, host): Section 3.3 and the metrics of Sections 5.2.2-5.2.4 ---------
__device__ __forceinline__ void start_cell(Ctx &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int slot, int host,
                                           int32_t now, int32_t start, int32_t t_submit, int32_t dur,
                                           uint32_t outcome) {
  int g = (int)((fl >> 3) & 7u) + 1;
  int32_t finish = start + dur;
  int32_t delay = start - t_submit;
  r.c_started++;
  r.sum_delay += delay;
  r.max_delay = r.max_delay > delay ? r.max_delay : delay;
  int b = delay == 0 ? 0 : 32 - __builtin_clz((uint32_t)delay);
  b = b > 31 ? 31 : b;
  if (c.lane == 0) atomicAdd(&c.m.hist[b], 1u);
  r.sum_tct += (int64_t)finish - t_submit;
  r.g_exec += (int64_t)g * dur;
  r.g_commit += (int64_t)g * ((int64_t)finish - now);
  uint32_t last = hw >> 30;                   // 0 none, else slot + 1
  if (last == (uint32_t)slot + 1u) r.reused++;
  hw = (hw & 0x3FFFFFFFu) | ((uint32_t)(slot + 1) << 30);
  hw = (hw & ~(1023u << (10 * slot))) | ((uint32_t)host << (10 * slot));
  uint32_t nfl = (fl & ~(7u | SF_QONCE | (15u << 8))) | SS_PLACED;
  if (c.lane == 0) {
    c.m.s_hosts[s] = hw;
    c.m.s_time[s] = finish;
    c.m.s_flag[s] = nfl;
  }
  r.lazy_max = r.lazy_max > finish ? r.lazy_max : finish;
  decide(c, r, now, outcome, s, (uint32_t)slot, (uint32_t)host);
  if (fl & SF_ENDING) queue_push(c, r, finish, QK_END, s, 0);
}

// ---- one attempt to run the pending cell of session s at time `now` -----------------------------
// hw / fl are the session's current words; retries is the number of retries already scheduled.
__device__ __forceinline__ void attempt(Ctx &c, Regs &r, uint32_t s, uint32_t hw, uint32_t fl, int32_t now,
                                        int32_t t_submit, int32_t dur) {
  wave_sync();
  const int G = c.p.G;
  int g = (int)((fl >> 3) & 7u) + 1;
  // (a) election, Section 3.2.2: lanes 0..23 = (replica r, GPU k) of the session's hosts
  int rr = c.lane >> 3, k = c.lane & 7;
  rr = rr > 2 ? 2 : rr;
  int hr = (int)((hw >> (10 * rr)) & 1023u);
  bool act = c.lane < 24 && k < G;
  int32_t f = c.m.fin[k * c.p.HP + hr];
  int32_t ra = c.m.ready_at[hr];
  uint64_t busy = wballot(act && f > now);
  uint64_t rdy = wballot(ra <= now);
  const int h0 = (int)(hw & 1023u), h1 = (int)((hw >> 10) & 1023u), h2 = (int)((hw >> 20) & 1023u);
  const int C0 = __builtin_popcount((uint32_t)busy & 0xFFu), C1 = __builtin_popcount((uint32_t)(busy >> 8) & 0xFFu),
            C2 = __builtin_popcount((uint32_t)(busy >> 16) & 0xFFu);
  const int ok0 = (int)(rdy & 1u), ok1 = (int)((rdy >> 8) & 1u), ok2 = (int)((rdy >> 16) & 1u);
  // feasible replica with the fewest committed GPUs, then the lowest host index
  const uint32_t k0 = (ok0 && G - C0 >= g) ? (((uint32_t)C0 << 12) | ((uint32_t)h0 << 2) | 0u) : 0xFFFFFFFFu;
  const uint32_t k1 = (ok1 && G - C1 >= g) ? (((uint32_t)C1 << 12) | ((uint32_t)h1 << 2) | 1u) : 0xFFFFFFFFu;
  const uint32_t k2 = (ok2 && G - C2 >= g) ? (((uint32_t)C2 << 12) | ((uint32_t)h2 << 2) | 2u) : 0xFFFFFFFFu;
  const uint32_t kb = umin(k0, umin(k1, k2));
  if (kb != 0xFFFFFFFFu) {
    const int lead = (int)(kb & 3u), hl = (int)((kb >> 2) & 1023u);
    int32_t finish = now + dur;
    bool fr = act && (c.lane >> 3) == lead && f <= now;
    int rank = lane_rank(wballot(fr));
    if (fr && rank < g) c.m.fin[k * c.p.HP + hr] = finish;
    if (now == t_submit) r.c_imm++;
    start_cell(c, r, s, hw, fl, lead, hl, now, now, t_submit, dur, NBOS_D_START);
    return;
  }
  // every replica yields: the replica on the fullest ready host would move (ties: lowest host).
  // Key: committed GPUs descending, host ascending -> minimise (8 - C, host).
  const int any_ready = ok0 | ok1 | ok2;
  const uint32_t v0 = (!any_ready || ok0) ? (((uint32_t)(8 - C0) << 12) | ((uint32_t)h0 << 2) | 0u) : 0xFFFFFFFFu;
  const uint32_t v1 = (!any_ready || ok1) ? (((uint32_t)(8 - C1) << 12) | ((uint32_t)h1 << 2) | 1u) : 0xFFFFFFFFu;
  const uint32_t v2 = (!any_ready || ok2) ? (((uint32_t)(8 - C2) << 12) | ((uint32_t)h2 << 2) | 2u) : 0xFFFFFFFFu;
  const uint32_t vb = umin(v0, umin(v1, v2));
  const int victim = (int)(vb & 3u), hv = (int)((vb >> 2) & 1023u);
  uint32_t moved = (uint32_t)g | (1u << 16);
  // (b) migration, Section 3.2.3: the target binds the GPUs at once. A ready host of this session
  // with g idle GPUs would have won the election, so none of its hosts can show up as a target.
  if (c.p.flags & NBOS_F_MIGRATE) {
    uint32_t key = best_host(c, now, g, true, -1, -1);
    if (key != 0xFFFFFFFFu) {
      int dst = (int)(key & 1023u);
      int32_t start = now + c.p.migr;
      if (c.lane == 0) { c.m.hsn[hv] -= moved; c.m.hsn[dst] += moved; }
      bind_gpus(c, dst, g, now, start + dur);
      r.migrations++;
      start_cell(c, r, s, hw, fl, victim, dst, now, start, t_submit, dur, NBOS_D_MIGRATE);
      return;
    }
  }
  // (c) a new host for the cell, Section 3.4.2: reserved and bound before it is up
  if ((c.p.flags & NBOS_F_SCALE_OUT) && r.n_on < c.p.Hmax) {
    int h = find_off_host(c);
    int32_t start = now + c.p.boot + c.p.migr;
    boot_host(c, r, h, now);
    if (c.lane == 0) { c.m.hsn[hv] -= moved; c.m.hsn[h] = moved; }
    bind_gpus(c, h, g, now, start + dur);
    r.so_hosts++;
    r.migrations++;
    start_cell(c, r, s, hw, fl, victim, h, now, start, t_submit, dur, NBOS_D_SCALE_CELL);
    return;
  }
  // (d) queue and retry periodically, then give up, Section 3.2.3
  int retries = (int)((fl >> 8) & 15u);
  if (retries < c.p.max_retries) {
    retries++;
    if (!(fl & SF_QONCE)) r.c_queued++;
    uint32_t nfl = (fl & ~(7u | (15u << 8))) | SS_QUEUED | SF_QONCE | ((uint32_t)retries << 8);
    if (c.lane == 0) { c.m.s_flag[s] = nfl; c.m.s_time[s] = t_submit; }
    queue_push(c, r, t_submit + retries * c.p.retry_iv, QK_RETRY, s, dur);
    return;
  }
  r.c_aborted++;
  decide(c, r, now, NBOS_D_ABORT, s, 0, 0);
  uint32_t nfl = (fl & ~(7u | SF_QONCE | (15u << 8))) | SS_PLACED;
  if (c.lane == 0) { c.m.s_flag[s] = nfl; c.m.s_time[s] = 0; }
  if (fl & SF_ENDING) end_session(c, r, s, hw, nfl, now);
}

// ---- the earliest queued timer fires ------------------------------------------------------------
__device__ __forceinline__ void queue_fire(Ctx &c, Regs &r) {
  wave_sync();
  int i = r.q_min_i;
  int32_t now = r.q_min_t;
  uint32_t key = uni(c.m.q_i[i]);
  int32_t dur = uni(c.m.q_d[i]);
  int last = r.q_n - 1;
  if (i != last) {                            // fill the hole with the last entry
    int32_t lt = c.m.q_t[last], ld = c.m.q_d[last];
    uint32_t li = c.m.q_i[last];
    if (c.lane == 0) { c.m.q_t[i] = lt; c.m.q_i[i] = li; c.m.q_d[i] = ld; }
  }
  r.q_n = last;
  r.t_end = r.t_end > now ? r.t_end : now;
  uint32_t s = key & 0xFFFFu;
  uint32_t hw = uni(c.m.s_hosts[s]), fl = uni(c.m.s_flag[s]);
  if ((key >> 16) == QK_RETRY) {
    int32_t t_submit = uni(c.m.s_time[s]);
    attempt(c, r, s, hw, fl, now, t_submit, dur);
  } else {
    end_session(c, r, s, hw, fl, now);
  }
  queue_rescan(c, r);
}

// ---- auto-scaler period: release at most two empty hosts (Section 3.4.2, last paragraph) --------
__device__ __forceinline__ void tick(Ctx &c, Regs &r, int32_t now) {
  wave_sync();
  int A = 0, Z = 0;
  for (int base = 0; base < c.p.HP; base += WAVE) {
    int h = base + c.lane;
    bool ready = c.m.ready_at[h] <= now;
    A += __builtin_popcountll(wballot(ready));
    Z += __builtin_popcountll(wballot(ready && (c.m.hsn[h] >> 16) == 0));
  }
  int released = 0;
  while ((int64_t)Z * 100 > (int64_t)A * c.p.idle_pct && A > c.p.min_hosts && released < 2) {
    int victim = -1;
    wave_sync();
    for (int base = c.p.HP - WAVE; base >= 0 && victim < 0; base -= WAVE) {
      int h = base + c.lane;
      uint64_t e = wballot(c.m.ready_at[h] <= now && (c.m.hsn[h] >> 16) == 0);
      if (e) victim = base + 63 - (int)__builtin_clzll(e);
    }
    if (c.lane == 0) c.m.ready_at[victim] = NEVER;
    r.n_on--;
    r.prov += (int64_t)c.p.G * now;
    A--; Z--; released++;
    r.si_hosts++;
    decide(c, r, now, NBOS_D_SCALE_IN, 0, 0, (uint32_t)victim);
  }
}

// ---- arrivals -----------------------------------------------------------------------------------
__device__ __forceinline__ void on_cell(Ctx &c, Regs &r, uint32_t s, int32_t now, int32_t dur) {
  wave_sync();
  r.c_total++;
  uint32_t fl = uni(c.m.s_flag[s]);
  uint32_t st = fl & 7u;
  if (st == SS_PLACED) {
    int32_t busy_until = uni(c.m.s_time[s]);
    if (busy_until > now) { r.c_busy++; return; }
    uint32_t hw = uni(c.m.s_hosts[s]);
    attempt(c, r, s, hw, fl & ~(SF_QONCE | (15u << 8)), now, now, dur);
  } else if (st == SS_QUEUED) {
    r.c_busy++;
  } else {
    r.c_unplaced++;
  }
}

__device__ __forceinline__ void on_session_end(Ctx &c, Regs &r, uint32_t s, int32_t now) {
  wave_sync();
  uint32_t fl = uni(c.m.s_flag[s]);
  uint32_t st = fl & 7u;
  if ((st != SS_PLACED && st != SS_QUEUED) || (fl & SF_ENDING)) return;
  int g = (int)((fl >> 3) & 7u) + 1;
  int32_t busy_until = uni(c.m.s_time[s]);
  r.open_g -= g;                              // the Reservation lifetime closes at the END event
  r.resv += (int64_t)g * now;
  if (st == SS_PLACED && busy_until <= now) {
    end_session(c, r, s, uni(c.m.s_hosts[s]), fl, now);
  } else {
    if (c.lane == 0) c.m.s_flag[s] = fl | SF_ENDING;
    if (st == SS_PLACED) queue_push(c, r, busy_until, QK_END, s, 0);
  }
}

// run every queued timer and auto-scaler period due at or before t
__device__ __forceinline__ void drain_until(Ctx &c, Regs &r, int32_t t, int32_t &tick_t) {
  const bool scale_in = (c.p.flags & NBOS_F_SCALE_IN) != 0;
  while (r.status == NBOS_OK) {
    bool q_due = r.q_n > 0 && r.q_min_t <= t;
    bool t_due = scale_in && tick_t <= t;
    if (q_due && (!t_due || r.q_min_t <= tick_t)) {
      queue_fire(c, r);
    } else if (t_due) {
      tick(c, r, tick_t);
      tick_t += c.p.scale_iv;
    } else {
      break;
    }
  }
}

__global__ void __launch_bounds__(WAVE) nbos_replay_lds_kernel(KParams p) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int rep = blockIdx.x;
  const int lane = threadIdx.x;
  if (rep >= p.n_replays) return;

  const int trace = p.trace_of_replay[rep];
  const int64_t ev_lo = p.ev_offset[trace], ev_hi = p.ev_offset[trace + 1];
  const int s_lo = p.sess_offset[trace];
  const int n_sess = p.sess_offset[trace + 1] - s_lo;

  // carve LDS
  Lds m;
  unsigned char *q = lds_raw;
  m.fin = (int32_t *)q;        q += (size_t)NGPU * p.HP * 4;
  m.ready_at = (int32_t *)q;   q += (size_t)p.HP * 4;
  m.hsn = (uint32_t *)q;       q += (size_t)p.HP * 4;
  m.hist = (uint32_t *)q;      q += 32 * 4;
  m.s_hosts = (uint32_t *)q;   q += (size_t)p.n_cap * 4;
  m.s_time = (int32_t *)q;     q += (size_t)p.n_cap * 4;
  m.s_flag = (uint32_t *)q;    q += (size_t)p.n_cap * 4;
  m.q_t = (int32_t *)q;        q += (size_t)p.q_cap * 4;
  m.q_i = (uint32_t *)q;       q += (size_t)p.q_cap * 4;
  m.q_d = (int32_t *)q;

  // S0: hosts 0..H0-1 ready at time 0, the rest off; sessions unplaced
  for (int i = lane; i < NGPU * p.HP; i += WAVE) m.fin[i] = 0;
  for (int h = lane; h < p.HP; h += WAVE) { m.ready_at[h] = h < p.H0 ? 0 : NEVER; m.hsn[h] = 0; }
  if (lane < 32) m.hist[lane] = 0;
  for (int s = lane; s < n_sess; s += WAVE) {
    uint32_t g = p.sess_gpus[s_lo + s];
    m.s_hosts[s] = 0; m.s_time[s] = 0; m.s_flag[s] = SS_UNPLACED | ((g - 1u) << 3);
  }
  __syncthreads();

  Ctx c{p, m, lane, p.cap_milli[rep] * p.G * 3, p.dlog ? p.dlog + (int64_t)rep * p.dlog_stride : nullptr};
  Regs r;
  memset(&r, 0, sizeof r);
  r.digest = 0xCBF29CE484222325ULL;
  r.n_on = p.H0;
  r.peak = (uint32_t)p.H0;
  r.q_min_t = NEVER;
  int32_t tick_t = p.scale_iv;
  int32_t t_last = 0;

  // S1: stream the events, one per lane per tile, next tile in flight
  int64_t base = ev_lo;
  int32_t vt = 0, vd = 0, vs = 0;
  if (base + lane < ev_hi) { vt = p.ev_time[base + lane]; vd = p.ev_dur[base + lane]; vs = p.ev_sk[base + lane]; }
  while (base < ev_hi && r.status == NBOS_OK) {
    int64_t nb = base + WAVE;
    int32_t nt = 0, nd = 0, ns = 0;
    if (nb + lane < ev_hi) { nt = p.ev_time[nb + lane]; nd = p.ev_dur[nb + lane]; ns = p.ev_sk[nb + lane]; }
    int cnt = (int)(ev_hi - base < WAVE ? ev_hi - base : WAVE);
    for (int i = 0; i < cnt && r.status == NBOS_OK; i++) {
      int32_t t = lane_get(vt, i), d = lane_get(vd, i);
      uint32_t sk = (uint32_t)lane_get(vs, i);
      uint32_t s = sk & 0xFFFFFFu, kind = sk >> 24;
      drain_until(c, r, t, tick_t);                       // S2
      t_last = t;
      if (kind == NBOS_EV_CELL) on_cell(c, r, s, t, d);    // S4-S8
      else if (kind == NBOS_EV_START) session_start(c, r, s, t);   // S3, S7
      else on_session_end(c, r, s, t);
    }
    vt = nt; vd = nd; vs = ns;
    base = nb;
  }

  // S10: drain. An auto-scaler period runs only while another timer is still pending.
  r.t_end = r.t_end > t_last ? r.t_end : t_last;
  const bool scale_in = (p.flags & NBOS_F_SCALE_IN) != 0;
  while (r.status == NBOS_OK) {
    if (r.q_n > 0) {
      if (scale_in && tick_t < r.q_min_t) { tick(c, r, tick_t); tick_t += p.scale_iv; }
      else queue_fire(c, r);
    } else if (scale_in && tick_t < r.lazy_max) {
      tick(c, r, tick_t); tick_t += p.scale_iv;
    } else {
      break;
    }
  }
  int32_t t_end = r.t_end > r.lazy_max ? r.t_end : r.lazy_max;
  r.prov += (int64_t)r.n_on * p.G * t_end;
  r.sub += (int64_t)r.sum_s * t_end;
  r.resv += (int64_t)r.open_g * t_end;

  __syncthreads();
  nbos_stats *out = p.stats + rep;
  if (lane < 32) out->delay_hist[lane] = m.hist[lane];
  if (lane == 0) {
    out->status = r.status; out->n_decisions = r.n_dec;
    out->sessions_placed = r.placed; out->sessions_rejected = r.rejected;
    out->cells_total = r.c_total; out->cells_immediate = r.c_imm; out->cells_started = r.c_started;
    out->cells_queued = r.c_queued; out->cells_aborted = r.c_aborted;
    out->cells_dropped_busy = r.c_busy; out->cells_dropped_unplaced = r.c_unplaced;
    out->executor_reused = r.reused; out->migrations = r.migrations;
    out->scale_out_hosts = r.so_hosts; out->scale_in_hosts = r.si_hosts; out->peak_hosts = r.peak;
    out->max_delay_ms = r.max_delay; out->t_end_ms = t_end;
    out->sum_delay_ms = r.sum_delay; out->sum_tct_ms = r.sum_tct;
    out->gpu_ms_executed = r.g_exec; out->gpu_ms_committed = r.g_commit;
    out->gpu_ms_provisioned = r.prov; out->reservation_gpu_ms = r.resv; out->sub_gpu_ms = r.sub;
    out->digest = r.digest;
  }
}

}  // namespace ldsk
}  // namespace
