// nbos_common.hpp — shared device helpers of the replay kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../include/nbos.h"

namespace {

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
  int32_t n_cap, q_cap;    // LDS capacity: sessions, queue entries
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
};

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

}  // namespace
