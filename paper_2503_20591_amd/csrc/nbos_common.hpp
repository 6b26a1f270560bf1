// nbos_common.hpp — shared device helpers of the replay kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../include/nbos.h"

namespace {

// ---- path profile (diagnostic build only: -DNBOS_PATH_PROFILE) -----------------------------------------
// Where does a replay spend its time? The wave that runs the replay reads the cycle counter at the marks
// below and adds the clocks since the previous mark to the category of the path just left (and a count);
// the sums of every replay go to a device array that nbos_path_profile_read copies out. The marks cost
// time of their own (two counter reads and two LDS atomics each), so a profiled launch runs about a tenth
// longer; the shares are what it is for. In the product build every mark is empty.
#ifdef NBOS_PATH_PROFILE
enum { PC_TILE, PC_ROUND, PC_ELECT, PC_MIGR, PC_FAIL, PC_START, PC_END, PC_TIMER_OTHER, PC_TICK, PC_RETRY_ELECT,
       PC_RETRY_MIGR, PC_RETRY_FAIL, PC_QUIET_RETRIES, PC_DROP, PC_LOOP_HORIZON, PC_LOOP_ROUND, PC_LOOP_TIMER,
       PC_LOOP_STARTEND, PC_LOOP_ATTEMPT, PC_HORIZON, PC_A_ELECT, PC_A_TARGET, PC_A_VICTIM, PC_A_BIND, PC_N };
constexpr int PATH_PROFILE_REPLAYS = 16384;      // replays beyond this many are not recorded
static __device__ unsigned long long g_path_profile[PATH_PROFILE_REPLAYS * 2 * PC_N];
__shared__ unsigned long long prof_t[PC_N];
__shared__ unsigned long long prof_n[PC_N];
#define PROF_BEGIN() if (threadIdx.x < PC_N) { prof_t[threadIdx.x] = 0; prof_n[threadIdx.x] = 0; } unsigned long long pt0 = __builtin_readcyclecounter()
#define PROF(cat, cnt) do { const unsigned long long now_ = __builtin_readcyclecounter(); if (threadIdx.x == 0) { atomicAdd(&prof_t[cat], now_ - pt0); atomicAdd(&prof_n[cat], (unsigned long long)(cnt)); } pt0 = __builtin_readcyclecounter(); } while (0)
// marks inside attempt(): clocks since the attempt began or since the mark before (these overlap PROF's)
#define PROF_SUB_BEGIN() unsigned long long pa0 = __builtin_readcyclecounter()
#define PROF_SUB(cat) do { const unsigned long long now_ = __builtin_readcyclecounter(); if (threadIdx.x == 0) { atomicAdd(&prof_t[cat], now_ - pa0); atomicAdd(&prof_n[cat], 1ull); } pa0 = __builtin_readcyclecounter(); } while (0)
#define PROF_OUT(rep) do { __syncthreads(); if (threadIdx.x < PC_N && (rep) < PATH_PROFILE_REPLAYS) { g_path_profile[((rep) * 2) * PC_N + threadIdx.x] = prof_t[threadIdx.x]; g_path_profile[((rep) * 2 + 1) * PC_N + threadIdx.x] = prof_n[threadIdx.x]; } } while (0)
// an attempt is booked by what came of it: the cell started by election, after a migration, or not at all
#define PROF_ATTEMPT_BEGIN(m, r) const uint32_t prof_st0 = (r).c_started; wave_sync(); const uint32_t prof_mg0 = uni((m).c32[CS_MIGR])
#define PROF_ATTEMPT_END(m, r, is_retry) do { wave_sync(); const uint32_t mg1_ = uni((m).c32[CS_MIGR]); \
    const int cat_ = (r).c_started == prof_st0 ? ((is_retry) ? PC_RETRY_FAIL : PC_FAIL) : mg1_ != prof_mg0 ? ((is_retry) ? PC_RETRY_MIGR : PC_MIGR) : ((is_retry) ? PC_RETRY_ELECT : PC_ELECT); \
    PROF(cat_, 1); } while (0)
#else
#define PROF_BEGIN() do { } while (0)
#define PROF(cat, cnt) do { } while (0)
#define PROF_SUB_BEGIN() do { } while (0)
#define PROF_SUB(cat) do { } while (0)
#define PROF_OUT(rep) do { } while (0)
#define PROF_ATTEMPT_BEGIN(m, r) do { } while (0)
#define PROF_ATTEMPT_END(m, r, is_retry) do { } while (0)
#endif

constexpr int WAVE = 64;
constexpr int32_t NEVER = 0x7FFFFFFF;
constexpr int NGPU = NBOS_MAX_GPUS;

// session states
constexpr uint32_t SS_UNPLACED = 0, SS_PLACED = 1, SS_QUEUED = 2, SS_REJECTED = 3, SS_ENDED = 4;
// session flag word: state[0..2] g-1[3..5] ending[6] queued_once[7] retries[8..11]
constexpr uint32_t SF_ENDING = 1u << 6, SF_QONCE = 1u << 7;
// queue entry kinds, in the order they run when due at the same time
constexpr uint32_t QK_END = 0, QK_RETRY = 2, QK_NEXT = 3;   // QK_NEXT: closed loop, the session's next event is due

struct KParams {
  const int64_t *ev_offset;
  const int32_t *ev_time, *ev_dur, *ev_sk;
  const int32_t *sess_offset;
  const uint8_t *sess_gpus;
  const int32_t *trace_of_replay, *cap_milli;
  nbos_stats *stats;
  uint64_t *dlog;          // null unless the decision log is on
  int32_t *ovf_dur;        // open loop: [n_replays][n_cap] durations of queued cells whose timer is
                           // outside the sorted registers
  int64_t dlog_stride;     // codes per replay
  int32_t n_replays, H0, Hmax, HP, G;
  uint32_t flags;
  int32_t migr, boot, retry_iv, max_retries, scale_iv, idle_pct, min_hosts;
  int32_t f_milli, buffer; // auto-scaler: f * 1000 of the expected capacity, extra hosts
  int32_t batch_delay;     // Batch baseline: container start per job
  int32_t warm_n, warm_migr, prewarm;   // pre-warmed containers per host, warm migration delay, pre-warm time
  int32_t n_cap;           // LDS capacity: sessions
  int32_t batch;           // event-parallel rounds on (LDS kernel)
  // closed loop only. cl_chain: per event of the traces {the next event of its session (index within
  // the trace, -1: none), the think time before that event}; the second word is -1 for an event no
  // chain holds. cl_cursor: per replay and session the event that is due next or under way.
  const int2 *cl_chain;
  int32_t *cl_cursor;
  // null, or a word a validation kernel of the same stream has left: when it is not 0 the traces are
  // invalid and every replay ends at once with status NBOS_E_RANGE (calls that cannot wait for the
  // validation on the host)
  const uint32_t *trace_err;
  // null, or the replay each workgroup runs (a permutation of 0..n_replays-1): the order of the launch
  const int32_t *order;
};

// Workgroups start in the order of their index, and consecutive ones go to different XCDs of the chip. The
// library therefore hands the replays out longest first (see order_replays in nbos_replay.hip): the heavy
// replays are spread over the XCDs and the short ones fill the tail of the launch.
__device__ __forceinline__ int launch_slot_replay(const KParams &p) {
  if ((int)blockIdx.x >= p.n_replays) return p.n_replays;       // (the callers return at once)
  return p.order ? p.order[blockIdx.x] : (int)blockIdx.x;
}

// A replay that cannot run (invalid traces, more sessions than the launch has LDS for): its record
// holds the status and zeros.
__device__ __forceinline__ void refuse_replay(const KParams &p, int rep, int lane, int32_t status) {
  int32_t *out = (int32_t *)(p.stats + rep);
  for (int i = lane; i < (int)(sizeof(nbos_stats) / 4); i += WAVE) out[i] = i == 0 ? status : 0;
}

__device__ __forceinline__ int32_t uni(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint32_t uni(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ int32_t lane_get(int32_t v, int l) { return __builtin_amdgcn_readlane(v, l); }

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// Minimum of v over the 64 lanes, returned wave-uniform. Four DPP butterfly steps make each row
// of 16 lanes uniform (quad swaps, half-row mirror, row mirror), then the four rows are combined
// on the scalar unit. Needs all lanes active.
__device__ __forceinline__ uint32_t wave_min(uint32_t v) {
  v = umin(v, dpp<0xB1>(v));    // quad_perm [1,0,3,2]
  v = umin(v, dpp<0x4E>(v));    // quad_perm [2,3,0,1]
  v = umin(v, dpp<0x141>(v));   // row_half_mirror
  v = umin(v, dpp<0x140>(v));   // row_mirror
  uint32_t a = (uint32_t)lane_get((int)v, 0), b = (uint32_t)lane_get((int)v, 16);
  uint32_t c = (uint32_t)lane_get((int)v, 32), d = (uint32_t)lane_get((int)v, 48);
  return umin(umin(a, b), umin(c, d));
}

// Lanes of the one wave talk through LDS (one lane writes, others read later). The hardware runs a
// wave's LDS operations in order; this only stops the compiler from keeping LDS values in registers
// or moving LDS accesses across the point. It emits no instruction.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// wave-wide ballot straight from the predicate (no int round trip)
__device__ __forceinline__ uint64_t wballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

__device__ __forceinline__ int lane_rank(uint64_t mask) {   // set bits of mask below this lane
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// ---- what the replay kernels share ---------------------------------------------------------------------
// Each kernel has its own context type C (the replay's parameters p, its LDS arrays m, the lane, the
// per-lane registers) and its own wave-uniform register block R; the helpers below work on either.

// Kernel instances: F is the set of policy flags when it is known at compile time (the common sets get
// an instance of their own, which drops the code of everything that is switched off), or one of the two
// values that leave the flags to run time.
constexpr uint32_t kRuntimeFlags = 0xFFFFFFFFu;
constexpr uint32_t kRuntimeClosed = 0xFFFFFFFEu;     // policy flags at run time, closed-loop reading of the trace
constexpr uint32_t kPolicyFlags = NBOS_F_MIGRATE | NBOS_F_SCALE_OUT | NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE | NBOS_F_DYNAMIC_SR |
                                  NBOS_F_STICKY_EXECUTOR | NBOS_F_WARM_POOL;
constexpr bool closed_loop_instance(uint32_t F) {
  return F == kRuntimeClosed || (F != kRuntimeFlags && (F & NBOS_F_CLOSED_LOOP) != 0);
}
template <uint32_t F>
__device__ __forceinline__ uint32_t instance_flags(const KParams &p) {
  return F == kRuntimeFlags ? (p.flags & ~NBOS_F_CLOSED_LOOP) : F == kRuntimeClosed ? (p.flags | NBOS_F_CLOSED_LOOP) : F;
}

// closed loop: a sorted timer's event has been loaded (bit 31 of qx); the widest refill window
constexpr int32_t CLX_LOADED = (int32_t)0x80000000;
constexpr int32_t CL_WIN_MAX = 1 << 24;

// Cold counters kept in LDS (lane 0 adds with ds_add, no return value). CS_BLAZY and the CL_B* sums are
// only fed by the event-parallel rounds of the any-size kernel.
enum { CS_PLACED, CS_REJECTED, CS_QUEUED, CS_ABORTED, CS_MIGR, CS_SO, CS_SI, CS_PEAK, CS_MAXDELAY,
       CS_NON, CS_SUMS, CS_OPENG, CS_BLAZY, CS_NREP, CS_MIGRWARM, CS_N32 };
enum { CL_SUMDELAY, CL_GWAIT, CL_PROV, CL_RESV, CL_SUB, CL_BDUR, CL_BGEXEC, CL_REPL, CL_N64 };

template <class L>
__device__ __forceinline__ void c32_add(L &m, int lane, int idx, uint32_t v) {
  if (lane == 0) atomicAdd(&m.c32[idx], v);
}
template <class L>
__device__ __forceinline__ void c32_max(L &m, int lane, int idx, uint32_t v) {
  if (lane == 0) atomicMax(&m.c32[idx], v);
}
template <class L>
__device__ __forceinline__ void c64_add(L &m, int lane, int idx, int64_t v) {
  if (lane == 0) atomicAdd(&m.c64[idx], (unsigned long long)v);
}

// Can the dynamic limit of Section 3.4.1 ever admit a host that the replay's own cap turns away? Not while
// every host that is on holds at most slim subscribed GPUs and more hosts are on than a request has GPUs:
// (S + g) n <= sum S + g <= n slim + g gives S + g <= slim + g / n, i.e. S + g <= slim for g < n. A host's
// S only grows through a placement or a migration that passed the limit (so S + g <= slim as long as the
// claim held so far) or starts at g on a host that was booted for the request (g <= G), so with slim >= G
// the claim holds for the whole replay, provided the cluster never has G hosts or fewer: it starts with
// H0 and the periodic release stops at min_hosts. Then the limit in force is the replay's cap, and the
// kernels keep the bounds that rest on a fixed cap. Otherwise (small clusters, caps below one request
// per empty host) the limit is worked out at every test.
__device__ __forceinline__ bool dynamic_limit_matters(const KParams &p, uint32_t flags, int32_t slim) {
  if (!(flags & NBOS_F_DYNAMIC_SR)) return false;
  const int32_t fewest = (flags & NBOS_F_SCALE_IN) ? (p.H0 < p.min_hosts ? p.H0 : p.min_hosts) : p.H0;
  return !(slim >= p.G && fewest > p.G);
}

// Largest S a host may hold and still take one more replica with request g (Section 3.4.1): the
// replay's cap, or with the dynamic limit the cluster-wide ratio after placing when that is larger:
// (S + g) / (G R) <= (sum S + g) / (n G R)  <=>  S + g <= floor((sum S + g) / n), n = hosts not off.
template <class C>
__device__ __forceinline__ int32_t cap_room(const C &c, int g) {
  int32_t lim = c.slim;
  if ((c.flags() & NBOS_F_DYNAMIC_SR) && c.dyn) {
    wave_sync();
    const uint32_t n_on = uni(c.m.c32[CS_NON]), tot = uni(c.m.c32[CS_SUMS]);
    if (n_on > 0) {
      const int32_t mean = (int32_t)((tot + (uint32_t)g) / n_on);
      lim = lim > mean ? lim : mean;
    }
  }
  return lim - g;
}

// One decision of the policy as a 64-bit code: host (10 bits), replica slot (2), outcome (4), session
// (16), time (32). The replay's digest is the FNV-style fold of its codes in order.
constexpr uint64_t DIGEST_PRIME = 0x100000001B3ULL;
__device__ __forceinline__ uint64_t decision_code(int32_t now, uint32_t outcome, uint32_t s, uint32_t slot,
                                                  uint32_t host) {
  return (uint64_t)host | ((uint64_t)slot << 10) | ((uint64_t)outcome << 12) | ((uint64_t)s << 16) |
         ((uint64_t)(uint32_t)now << 32);
}
template <class C, class R>
__device__ __forceinline__ void decide(C &c, R &r, int32_t now, uint32_t outcome, uint32_t s, uint32_t slot,
                                       uint32_t host) {
  const uint64_t code = decision_code(now, outcome, s, slot, host);
  r.digest = r.digest * DIGEST_PRIME + code;
  if (__builtin_expect(c.dlog != nullptr, 0)) {
    if (c.lane == 0 && (int64_t)r.n_dec < c.p.dlog_stride) c.dlog[r.n_dec] = code;
  }
  r.n_dec++;
}

// ---- timers: the 64 earliest, sorted ascending by (time, kind << 16 | id), entry i in lane i -----
// Invariant: every entry in the registers is earlier than every timer that waits in the session
// records, and the registers are empty only if none waits there. Each kernel brings its own
// ovf_push (a timer goes to wait in its session's record) and refill (the earliest waiting timers come
// into the registers).
template <class C, class R>
__device__ __forceinline__ void timer_push(C &c, R &r, int32_t t, uint32_t kind, uint32_t id, int32_t d,
                                           int32_t x = 0, int32_t nx = -1, int32_t nth = 0) {
  uint32_t k = (kind << 16) | id;
  if (__builtin_expect(r.q_n == WAVE, 0)) {
    int32_t mt = lane_get(c.qt, WAVE - 1);
    uint32_t mk = (uint32_t)lane_get((int)c.qk, WAVE - 1);
    if (t < mt || (t == mt && k < mk)) {
      ovf_push(c, r, mt, mk, lane_get(c.qd, WAVE - 1));   // the latest register entry moves out
      r.q_n = WAVE - 1;
    } else {
      ovf_push(c, r, t, k, d);
      return;
    }
  } else if (r.o_n > 0 && !(t < r.o_min_t || (t == r.o_min_t && k < r.o_min_k))) {
    ovf_push(c, r, t, k, d);
    return;
  }
  bool before = c.lane < r.q_n && (c.qt < t || (c.qt == t && c.qk < k));
  int pos = __builtin_popcountll(wballot(before));
  int32_t st = __builtin_amdgcn_update_dpp(c.qt, c.qt, 0x138, 0xF, 0xF, false);          // wave_shr:1
  int32_t sd = __builtin_amdgcn_update_dpp(c.qd, c.qd, 0x138, 0xF, 0xF, false);
  uint32_t sk = (uint32_t)__builtin_amdgcn_update_dpp((int)c.qk, (int)c.qk, 0x138, 0xF, 0xF, false);
  if (c.lane > pos) { c.qt = st; c.qd = sd; c.qk = sk; }
  if (c.lane == pos) { c.qt = t; c.qd = d; c.qk = k; }
  if constexpr (C::closed) {
    const int32_t sx = __builtin_amdgcn_update_dpp(c.qx, c.qx, 0x138, 0xF, 0xF, false);
    const int32_t sn = __builtin_amdgcn_update_dpp(c.qnx, c.qnx, 0x138, 0xF, 0xF, false);
    const int32_t sh = __builtin_amdgcn_update_dpp(c.qnth, c.qnth, 0x138, 0xF, 0xF, false);
    if (c.lane > pos) { c.qx = sx; c.qnx = sn; c.qnth = sh; }
    if (c.lane == pos) { c.qx = x; c.qnx = nx; c.qnth = nth; }
  }
  r.q_n++;
  if (pos == 0) r.q_head_t = t;
}

// remove the earliest timer (lane 0); refill from the session records when the registers run empty
template <class C, class R>
__device__ __forceinline__ void timer_pop(C &c, R &r) {
  c.qt = __builtin_amdgcn_update_dpp(c.qt, c.qt, 0x130, 0xF, 0xF, false);                // wave_shl:1
  c.qd = __builtin_amdgcn_update_dpp(c.qd, c.qd, 0x130, 0xF, 0xF, false);
  c.qk = (uint32_t)__builtin_amdgcn_update_dpp((int)c.qk, (int)c.qk, 0x130, 0xF, 0xF, false);
  r.q_n--;
  if constexpr (C::closed) {
    c.qx = __builtin_amdgcn_update_dpp(c.qx, c.qx, 0x130, 0xF, 0xF, false);
    c.qnx = __builtin_amdgcn_update_dpp(c.qnx, c.qnx, 0x130, 0xF, 0xF, false);
    c.qnth = __builtin_amdgcn_update_dpp(c.qnth, c.qnth, 0x130, 0xF, 0xF, false);
  }
  if (__builtin_expect(r.q_n == 0 && r.o_n > 0, 0)) refill(c, r);
  r.q_head_t = r.q_n > 0 ? lane_get(c.qt, 0) : NEVER;
}

}  // namespace
