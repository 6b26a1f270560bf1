// nbos_replay.hip — batched NotebookOS policy replay for gfx950 (MI355X): C ABI, input validation
// and kernel dispatch. Two kernels implement the same replay (see their headers):
//   nbos_kernel_reg.hpp   hosts_max <= 64: host state in registers, no LDS round trip per cell
//   nbos_kernel_lds.hpp   any hosts_max up to 1024: host state in LDS
// A third replays the Batch baseline policy on the same traces (nbos_kernel_batch.hpp); the traces are
// read as closed loops by a variant of either kernel (the end of nbos_kernel_reg.hpp, nbos_kernel_closed.hpp).
// Everything is integer arithmetic; all control flow is wave-uniform.

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/nbos.h"
#include "nbos_common.hpp"
#include "nbos_kernel_lds.hpp"
#include "nbos_kernel_closed.hpp"
#include "nbos_kernel_reg.hpp"
#include "nbos_kernel_batch.hpp"

namespace {

// ---- input validation (device side: the traces are device memory) -------------------------------
// err bits: 1 time order / sign, 2 time overflow, 4 kind, 8 session id, 16 duration, 32 GPU request,
// 64 trace index, 128 cap
__device__ __forceinline__ void validate_trace_body(const int64_t *ev_offset, const int32_t *ev_time, const int32_t *ev_dur,
                                                    const int32_t *ev_sk, const int32_t *sess_offset,
                                                    const uint8_t *sess_gpus, int G, int32_t t_limit, uint32_t *err) {
  int trace = blockIdx.x;
  int64_t lo = ev_offset[trace], hi = ev_offset[trace + 1];
  int s_lo = sess_offset[trace], n_sess = sess_offset[trace + 1] - s_lo;
  uint32_t e = 0;
  for (int64_t i = lo + threadIdx.x; i < hi; i += blockDim.x) {
    int32_t t = ev_time[i];
    uint32_t sk = (uint32_t)ev_sk[i];
    uint32_t kind = sk >> 24, s = sk & 0xFFFFFFu;
    if (t < 0 || (i > lo && ev_time[i - 1] > t)) e |= 1;
    if (t > t_limit) e |= 2;
    if (kind > NBOS_EV_END) e |= 4;
    if (s >= (uint32_t)n_sess) e |= 8;
    if (kind == NBOS_EV_CELL && (ev_dur[i] < 1 || ev_dur[i] > NBOS_MAX_DUR_MS)) e |= 16;
  }
  for (int s = threadIdx.x; s < n_sess; s += blockDim.x) {
    int g = sess_gpus[s_lo + s];
    if (g < 1 || g > G) e |= 32;
  }
  if (e) atomicOr(err, e);
}

__global__ void nbos_validate_traces(const int64_t *ev_offset, const int32_t *ev_time, const int32_t *ev_dur,
                                     const int32_t *ev_sk, const int32_t *sess_offset, const uint8_t *sess_gpus,
                                     int G, int32_t t_limit, uint32_t *err) {
  validate_trace_body(ev_offset, ev_time, ev_dur, ev_sk, sess_offset, sess_gpus, G, t_limit, err);
}

// the same after nbos_validate_offsets on the same stream: traces are only walked if their offsets are sound
__global__ void nbos_validate_traces_checked(const int64_t *ev_offset, const int32_t *ev_time, const int32_t *ev_dur,
                                             const int32_t *ev_sk, const int32_t *sess_offset, const uint8_t *sess_gpus,
                                             int G, int32_t t_limit, uint32_t *err) {
  if (*err & 256u) return;
  validate_trace_body(ev_offset, ev_time, ev_dur, ev_sk, sess_offset, sess_gpus, G, t_limit, err);
}

__global__ void nbos_validate_replays(const int32_t *trace_of_replay, const int32_t *cap_milli, int n_replays,
                                      int n_traces, uint32_t *err) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_replays) return;
  uint32_t e = 0;
  if (trace_of_replay[i] < 0 || trace_of_replay[i] >= n_traces) e |= 64;
  if (cap_milli[i] < 1 || cap_milli[i] > NBOS_MAX_CAP_MILLI) e |= 128;
  if (e) atomicOr(err, e);
}

// ---- scratch memory of the entry point that allocates nothing ----------------------------------------
// Word 0: the error bits of the validation kernels; from word 64 on: the register kernel's array of
// queued durations, [n_replays][sessions per trace]. One copy per GPU, held until the process ends.
constexpr size_t kScratchWords = 4u * 1024u * 1024u;              // 16 MiB
constexpr size_t kScratchHead = 64;
static __device__ __align__(256) int32_t scratch[kScratchWords];

__global__ void nbos_clear_word(uint32_t *w) { *w = 0u; }

// offsets of the traces, checked on the device for callers that cannot wait for a copy: err bit 256
__global__ void nbos_validate_offsets(const int64_t *ev_offset, const int32_t *sess_offset, int n_traces, uint32_t *err) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t > n_traces) return;
  uint32_t e = 0;
  if (t == 0 && (ev_offset[0] != 0 || sess_offset[0] != 0)) e |= 256;
  if (t < n_traces && (ev_offset[t + 1] < ev_offset[t] || sess_offset[t + 1] < sess_offset[t])) e |= 256;
  if (e) atomicOr(err, e);
}

// the register kernel for nj = ceil(hosts_max / 8) groups of 8 hosts and a compile-time flag set
template <uint32_t F>
const void *reg_kernel_for(int nj) {
  switch (nj) {
    case 1: return (const void *)regk::nbos_replay_reg_kernel<1, F>;
    case 2: return (const void *)regk::nbos_replay_reg_kernel<2, F>;
    case 3: return (const void *)regk::nbos_replay_reg_kernel<3, F>;
    case 4: return (const void *)regk::nbos_replay_reg_kernel<4, F>;
    case 5: return (const void *)regk::nbos_replay_reg_kernel<5, F>;
    case 6: return (const void *)regk::nbos_replay_reg_kernel<6, F>;
    case 7: return (const void *)regk::nbos_replay_reg_kernel<7, F>;
    default: return (const void *)regk::nbos_replay_reg_kernel<8, F>;
  }
}

// the same for the closed-loop reading of the traces
template <uint32_t F>
const void *reg_closed_kernel_for(int nj) {
  switch (nj) {
    case 1: return (const void *)regk::nbos_replay_reg_closed_kernel<1, F>;
    case 2: return (const void *)regk::nbos_replay_reg_closed_kernel<2, F>;
    case 3: return (const void *)regk::nbos_replay_reg_closed_kernel<3, F>;
    case 4: return (const void *)regk::nbos_replay_reg_closed_kernel<4, F>;
    case 5: return (const void *)regk::nbos_replay_reg_closed_kernel<5, F>;
    case 6: return (const void *)regk::nbos_replay_reg_closed_kernel<6, F>;
    case 7: return (const void *)regk::nbos_replay_reg_closed_kernel<7, F>;
    default: return (const void *)regk::nbos_replay_reg_closed_kernel<8, F>;
  }
}

// ---- billing post-pass (the paper's "Monetary Cost" section): one lane per replay ---------------------------------
// floor(a * b / d) for a, b, d below 2^63 with a quotient below 2^64: 128-bit product, then binary
// long division (the remainder stays below d, so it never overflows when doubled)
__device__ uint64_t muldiv_floor(uint64_t a, uint64_t b, uint64_t d) {
  const uint64_t hi = __umul64hi(a, b), lo = a * b;
  uint64_t rem = 0, q = 0;
  for (int i = 127; i >= 0; --i) {
    const uint64_t bit = i >= 64 ? (hi >> (i - 64)) & 1u : (lo >> i) & 1u;
    rem = (rem << 1) | bit;
    q <<= 1;
    if (rem >= d) { rem -= d; q |= 1u; }
  }
  return q;
}

__global__ void nbos_billing_kernel(const nbos_stats *stats, int first, int count, int G, int64_t price,
                                    int32_t markup_pct, int32_t standby_permille, nbos_bill *out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const nbos_stats &s = stats[first + i];
  const uint64_t ms_per_hour = 3600000u;
  const uint64_t exec_ms = (uint64_t)(s.sum_tct_ms - s.sum_delay_ms);      // every started cell runs its duration
  // no replicas (Batch baseline): nothing stands by
  const uint64_t standby_ms = (uint64_t)s.replica_ms > exec_ms ? (uint64_t)s.replica_ms - exec_ms : 0u;
  const uint64_t marked = (uint64_t)price * (uint64_t)markup_pct;
  nbos_bill b;
  b.provider_cost = (int64_t)muldiv_floor((uint64_t)s.gpu_ms_provisioned, (uint64_t)price, (uint64_t)G * ms_per_hour);
  b.usage_revenue = (int64_t)muldiv_floor((uint64_t)s.gpu_ms_executed, marked, (uint64_t)G * ms_per_hour * 100u);
  b.standby_revenue = (int64_t)muldiv_floor(standby_ms, marked * (uint64_t)standby_permille, ms_per_hour * 100000u);
  b.reservation_revenue = (int64_t)muldiv_floor((uint64_t)s.reservation_gpu_ms, marked, (uint64_t)G * ms_per_hour * 100u);
  out[i] = b;
}

// ---- measurement aid: the dependency-chain floor of one event body ---------------------------------
// A replay is a serial chain: an event cannot begin before the previous one's state update. The
// shortest such step this design can take is: read one host's GPU row from LDS, count the committed
// GPUs, one wave-wide minimum over a packed key, write one busy-until time back. The kernel runs that
// body `iters` times in a dependent chain (the minimum picks the next host), one wave per workgroup
// on its own SIMD; time / iters is the floor a replay's ns-per-event figure is compared with.
__global__ void __launch_bounds__(WAVE) nbos_chain_floor_kernel(int iters, uint32_t *sink) {
  __shared__ int4 rows[2 * WAVE];
  const int lane = threadIdx.x;
  rows[2 * lane] = make_int4(lane, 2 * lane, 3, 5);
  rows[2 * lane + 1] = make_int4(7, lane ^ 21, 11, 13);
  __syncthreads();
  int h = lane;
  int32_t now = 0;
  uint32_t acc = blockIdx.x;
  for (int i = 0; i < iters; i++) {
    wave_sync();
    const int4 a = rows[2 * h], b = rows[2 * h + 1];
    const int C = (a.x > now) + (a.y > now) + (a.z > now) + (a.w > now) + (b.x > now) + (b.y > now) + (b.z > now) + (b.w > now);
    const uint32_t key = ((uint32_t)C << 22) | (((uint32_t)lane * 2654435761u + acc) & 0x3FFFC0u) | (uint32_t)lane;
    const uint32_t m = wave_min(key);
    h = (int)(m & 63u);
    if (lane == 0) rows[2 * h].x = now + 1 + (int32_t)((m >> 6) & 7u);
    now += 1;
    acc = m;
    h = (h + lane) & 63;
  }
  if (lane == 0) sink[blockIdx.x] = acc;
}

}  // namespace

// ================================= host side: the C ABI ===========================================

struct nbos_replay {
  nbos_config cfg;
  nbos_inputs in;
  hipStream_t stream;
  int device;
  KParams kp;
  size_t lds_bytes;
  int threads;             // per workgroup: one wave, or four on large clusters (three helper waves for the scans)
  const void *kernel;      // the kernel instance chosen at create
  char kernel_name[96];    // as a profiler prints it, without the argument list
  nbos_stats *d_stats;
  nbos_bill *d_bill;
  int32_t *d_ovf;          // open-loop replay kernels: durations of queued cells, [n_replays][n_cap]
  int32_t *d_order;        // the replay each workgroup of the launch runs
  int32_t *d_chain;        // closed loop only: the chain records of all events, then the cursors
  uint64_t *d_log;
  std::vector<int64_t> ev_off;
  std::vector<int32_t> sess_off;
  std::vector<int32_t> trace_of_replay;   // only with the decision log
  hipEvent_t e0, e1;
  bool ran;
};

namespace {
void free_handle(nbos_replay *h) {
  if (!h) return;
  if (h->d_stats) (void)hipFree(h->d_stats);
  if (h->d_bill) (void)hipFree(h->d_bill);
  if (h->d_ovf) (void)hipFree(h->d_ovf);
  if (h->d_order) (void)hipFree(h->d_order);
  if (h->d_chain) (void)hipFree(h->d_chain);
  if (h->d_log) (void)hipFree(h->d_log);
  if (h->e0) (void)hipEventDestroy(h->e0);
  if (h->e1) (void)hipEventDestroy(h->e1);
  delete h;
}

// ---- steps of nbos_replay_create -------------------------------------------------------------------
// what nbos_last_error_detail() returns on this thread: the runtime call that failed and the runtime's word for it
thread_local char g_detail[256] = "";
void note_hip_failure(const char *call, hipError_t e) {
  snprintf(g_detail, sizeof g_detail, "%s: %s", call, hipGetErrorString(e));
}
#define HIP_TRY(x) do { const hipError_t e_ = (x); if (e_ != hipSuccess) { note_hip_failure(#x, e_); return NBOS_E_HIP; } } while (0)

// the configuration in the current layout (earlier, shorter layouts are accepted: later fields read as 0)
int32_t read_config(const nbos_config *cfg_in, nbos_config *full) {
  constexpr uint32_t kShortConfig = offsetof(nbos_config, autoscale_f_milli);
  constexpr uint32_t kMidConfig = offsetof(nbos_config, batch_start_delay_ms);
  constexpr uint32_t kBatchConfig = offsetof(nbos_config, warm_pool_per_host);
  if (cfg_in->struct_size != sizeof(nbos_config) && cfg_in->struct_size != kShortConfig &&
      cfg_in->struct_size != kMidConfig && cfg_in->struct_size != kBatchConfig)
    return NBOS_E_ARG;
  memset(full, 0, sizeof *full);
  memcpy(full, cfg_in, cfg_in->struct_size);
  full->struct_size = sizeof(nbos_config);
  return NBOS_OK;
}

// host-side checks of the parameters
int32_t check_config(const nbos_config *cfg, const nbos_inputs *in) {
  if (cfg->n_replays < 0 || cfg->n_traces < 0 || (cfg->n_replays > 0 && cfg->n_traces < 1)) return NBOS_E_ARG;
  if (cfg->replicas != 3) return NBOS_E_ARG;
  if (cfg->gpus_per_host < 1 || cfg->gpus_per_host > NBOS_MAX_GPUS) return NBOS_E_ARG;
  if (cfg->hosts_initial < 1 || cfg->hosts_max < cfg->hosts_initial) return NBOS_E_ARG;
  if (cfg->hosts_max > NBOS_MAX_HOSTS) return NBOS_E_LIMIT;
  if (cfg->migration_delay_ms < 0 || cfg->boot_delay_ms < 0 || cfg->retry_interval_ms < 1) return NBOS_E_ARG;
  if (cfg->max_retries < 0 || cfg->max_retries > NBOS_MAX_RETRIES) return NBOS_E_ARG;
  constexpr uint32_t kComparison = NBOS_F_HOSTS_IN_LDS | NBOS_F_GENERIC_KERNEL | NBOS_F_ROUNDS_OFF | NBOS_F_ROUNDS_ON |
                                   NBOS_F_ONE_WAVE;
  if (cfg->flags & ~(NBOS_F_MIGRATE | NBOS_F_SCALE_OUT | NBOS_F_SCALE_IN | NBOS_F_DECISION_LOG | kComparison |
                     NBOS_F_AUTOSCALE | NBOS_F_DYNAMIC_SR | NBOS_F_STICKY_EXECUTOR | NBOS_F_BATCH_MODE | NBOS_F_WARM_POOL |
                     NBOS_F_CLOSED_LOOP))
    return NBOS_E_ARG;
  if ((cfg->flags & NBOS_F_ROUNDS_OFF) && (cfg->flags & NBOS_F_ROUNDS_ON)) return NBOS_E_ARG;
  if ((cfg->flags & NBOS_F_CLOSED_LOOP) && (cfg->flags & (NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE | NBOS_F_BATCH_MODE)))
    return NBOS_E_ARG;
  if (cfg->flags & NBOS_F_WARM_POOL) {
    if (cfg->warm_pool_per_host < 1 || cfg->warm_pool_per_host > 4 || cfg->warm_migration_delay_ms < 0 ||
        cfg->prewarm_delay_ms < 0 || cfg->prewarm_delay_ms > NBOS_MAX_DUR_MS)
      return NBOS_E_ARG;
  }
  if (cfg->flags & NBOS_F_BATCH_MODE) {
    if (cfg->flags & ~(NBOS_F_BATCH_MODE | NBOS_F_SCALE_OUT | NBOS_F_DECISION_LOG | kComparison)) return NBOS_E_ARG;   // no pool either
    if (cfg->batch_start_delay_ms < 0 || cfg->batch_start_delay_ms > NBOS_MAX_DUR_MS) return NBOS_E_ARG;
  }
  if (cfg->flags & (NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE)) {
    if (cfg->scale_interval_ms < 1 || cfg->min_hosts < 0) return NBOS_E_ARG;
  }
  if (cfg->flags & NBOS_F_SCALE_IN) {
    if (cfg->scale_in_idle_pct < 0 || cfg->scale_in_idle_pct > 100) return NBOS_E_ARG;
  }
  if (cfg->flags & NBOS_F_AUTOSCALE) {
    if (cfg->autoscale_f_milli < 0 || cfg->autoscale_f_milli > 100000) return NBOS_E_ARG;
    if (cfg->scaling_buffer_hosts < 0 || cfg->scaling_buffer_hosts > NBOS_MAX_HOSTS) return NBOS_E_ARG;
  }
  if (cfg->n_replays > 0 &&
      (!in->ev_offset || !in->sess_offset || !in->trace_of_replay || !in->cap_milli)) return NBOS_E_ARG;
  return NBOS_OK;
}

// the time a replay can reach beyond its last arrival
int64_t time_slack(const nbos_config *cfg) {
  int64_t slowest = cfg->migration_delay_ms;
  if ((cfg->flags & NBOS_F_WARM_POOL) && cfg->warm_migration_delay_ms > slowest) slowest = cfg->warm_migration_delay_ms;
  // the auto-scaler's next period is scheduled one interval past the last instant that matters
  const int64_t period = (cfg->flags & (NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE)) ? cfg->scale_interval_ms : 0;
  return (int64_t)NBOS_MAX_DUR_MS + (int64_t)cfg->max_retries * cfg->retry_interval_ms + cfg->boot_delay_ms + slowest +
         ((cfg->flags & NBOS_F_WARM_POOL) ? cfg->prewarm_delay_ms : 0) + period;
}

int32_t open_device(nbos_replay *h) {
  HIP_TRY(hipGetDevice(&h->device));
  HIP_TRY(hipEventCreate(&h->e0));
  HIP_TRY(hipEventCreate(&h->e1));
  return NBOS_OK;
}

// what create works out about the batch before it chooses a kernel
struct Shape {
  int32_t max_sess = 0;     // most sessions in one trace
  int64_t max_ev = 0;       // most events in one trace
  int64_t total_ev = 0;
  int HP = 0;               // hosts_max rounded up to whole waves
  int n_cap = 1;            // session capacity of a replay's LDS
  bool in_regs = false;     // the register kernel runs
};

// the offsets of the traces, copied to the host
int32_t read_offsets(nbos_replay *h, Shape *sh) {
  const nbos_config *cfg = &h->cfg;
  const nbos_inputs *in = &h->in;
  const int nt = cfg->n_traces;
  if (cfg->n_replays == 0) return NBOS_OK;
  h->ev_off.resize((size_t)nt + 1);
  h->sess_off.resize((size_t)nt + 1);
  HIP_TRY(hipMemcpyAsync(h->ev_off.data(), in->ev_offset, sizeof(int64_t) * (nt + 1), hipMemcpyDeviceToHost, h->stream));
  HIP_TRY(hipMemcpyAsync(h->sess_off.data(), in->sess_offset, sizeof(int32_t) * (nt + 1), hipMemcpyDeviceToHost, h->stream));
  HIP_TRY(hipStreamSynchronize(h->stream));
  if (h->ev_off[0] != 0 || h->sess_off[0] != 0) return NBOS_E_RANGE;
  for (int t = 0; t < nt; t++) {
    const int64_t ne = h->ev_off[t + 1] - h->ev_off[t];
    const int64_t ns = (int64_t)h->sess_off[t + 1] - h->sess_off[t];
    if (ne < 0 || ns < 0) return NBOS_E_RANGE;
    if (ns > NBOS_MAX_SESSIONS) return NBOS_E_LIMIT;
    if ((cfg->flags & NBOS_F_CLOSED_LOOP) && ne >= 0x40000000LL) return NBOS_E_LIMIT;    // event indices within a trace
    if (ns > sh->max_sess) sh->max_sess = (int32_t)ns;
    if (ne > sh->max_ev) sh->max_ev = ne;
  }
  sh->total_ev = h->ev_off[nt];
  if ((sh->total_ev > 0 && (!in->ev_time_ms || !in->ev_dur_ms || !in->ev_sess_kind)) ||
      (h->sess_off[nt] > 0 && !in->sess_gpus))
    return NBOS_E_ARG;
  return NBOS_OK;
}

// the kernel instance a handle launches, with its name as a profiler prints it
void set_kernel(nbos_replay *h, const void *k, const char *fmt, int a, uint32_t f) {
  h->kernel = k;
  if (a >= 0) snprintf(h->kernel_name, sizeof h->kernel_name, fmt, a, (unsigned)f);
  else snprintf(h->kernel_name, sizeof h->kernel_name, fmt, (unsigned)f);
}
template <uint32_t F> void set_lds_kernel(nbos_replay *h) {
  set_kernel(h, (const void *)ldsk::nbos_replay_lds_kernel<F>, "ldsk::nbos_replay_lds_kernel<%uu>", -1, F);
}
template <uint32_t F> void set_closed_kernel(nbos_replay *h) {
  set_kernel(h, (const void *)ldsk::nbos_replay_closed_kernel<F>, "ldsk::nbos_replay_closed_kernel<%uu>", -1, F);
}
template <uint32_t F> void set_reg_closed_kernel(nbos_replay *h, int nj) {
  set_kernel(h, reg_closed_kernel_for<F>(nj), "regk::nbos_replay_reg_closed_kernel<%d, %uu>", nj > 8 ? 8 : nj, F);
}

// which flavour of the register kernel: see the comment inside
int32_t choose_reg_kernel(nbos_replay *h, int maxlds) {
  const nbos_config *cfg = &h->cfg;
  // The common policy flag sets have kernels compiled for them (everything that is switched off
  // is gone from the code): the shorter path per item makes them faster at every occupancy the
  // kernels reach (both are compiled for at most 128 registers, i.e. up to 16 workgroups per
  // compute unit; measured: 30 hosts, 4 per compute unit, -10 %; 64 hosts, 16 per compute unit,
  // 288 against 307 ms; 24 hosts, 64 per compute unit in four rounds, 100 against 115 ms). The
  // generic kernel runs for the other flag sets, and if it ever needs fewer rounds for the batch
  // (a batch that does not fit at once runs in rounds; waves hide little of each other's latency).
  const int nj = (cfg->hosts_max + 7) / 8;
  const uint32_t policy = cfg->flags & kPolicyFlags;
  const void *generic = reg_kernel_for<kRuntimeFlags>(nj);
  const bool has_special = policy == 0u || policy == NBOS_F_MIGRATE || policy == (NBOS_F_MIGRATE | NBOS_F_SCALE_OUT);
  const void *special = policy == 0u ? reg_kernel_for<0u>(nj)
                      : policy == NBOS_F_MIGRATE ? reg_kernel_for<NBOS_F_MIGRATE>(nj)
                      : policy == (NBOS_F_MIGRATE | NBOS_F_SCALE_OUT) ? reg_kernel_for<NBOS_F_MIGRATE | NBOS_F_SCALE_OUT>(nj)
                      : generic;
  int cus = 0;
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device));
  bool use_generic;
  if (cfg->flags & NBOS_F_GENERIC_KERNEL) {                 // comparison runs
    use_generic = true;
  } else {
    const int per_cu = cus > 0 ? (cfg->n_replays + cus - 1) / cus : cfg->n_replays;
    hipFuncAttributes fa_g, fa_s;
    HIP_TRY(hipFuncGetAttributes(&fa_g, generic));
    HIP_TRY(hipFuncGetAttributes(&fa_s, special));
    const int by_lds = (int)((size_t)maxlds / ((h->lds_bytes + 511) / 512 * 512));
    auto resident = [&](const hipFuncAttributes &fa) {      // workgroups (= waves) per compute unit
      const int regs = (fa.numRegs + 7) / 8 * 8;
      int per_simd = regs > 0 ? 512 / regs : 8;
      per_simd = per_simd > 8 ? 8 : per_simd;
      const int by_regs = 4 * per_simd;
      return by_lds < by_regs ? by_lds : by_regs;
    };
    const int res_g = resident(fa_g) > 0 ? resident(fa_g) : 1, res_s = resident(fa_s) > 0 ? resident(fa_s) : 1;
    use_generic = (per_cu + res_g - 1) / res_g < (per_cu + res_s - 1) / res_s;
  }
  if (use_generic || !has_special) set_kernel(h, generic, "regk::nbos_replay_reg_kernel<%d, %uu>", nj, kRuntimeFlags);
  else set_kernel(h, special, "regk::nbos_replay_reg_kernel<%d, %uu>", nj, policy);
  return NBOS_OK;
}

// kernel choice and LDS footprint of one replay
int32_t choose_kernel(nbos_replay *h, Shape *sh) {
  const nbos_config *cfg = &h->cfg;
  const bool batch_mode = (cfg->flags & NBOS_F_BATCH_MODE) != 0, warm_pool = (cfg->flags & NBOS_F_WARM_POOL) != 0;
  const bool closed_loop = (cfg->flags & NBOS_F_CLOSED_LOOP) != 0;
  int maxlds = 0;
  HIP_TRY(hipDeviceGetAttribute(&maxlds, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device));
#ifdef NBOS_PATH_PROFILE
  maxlds -= 2 * 8 * PC_N;                   // the profile's own counters are static LDS
#endif
  sh->in_regs = cfg->hosts_max <= WAVE && !(cfg->flags & NBOS_F_HOSTS_IN_LDS) && !batch_mode && !closed_loop;
  sh->HP = (cfg->hosts_max + WAVE - 1) / WAVE * WAVE;
  // the kernels with host state in LDS give the scans over all hosts to four waves from 256 hosts on
  h->threads = (!sh->in_regs && !batch_mode && sh->HP >= 4 * WAVE && !(cfg->flags & NBOS_F_ONE_WAVE)) ? ldsk::MAX_WAVES * WAVE : WAVE;
  sh->n_cap = sh->max_sess > 0 ? sh->max_sess : 1;
  const int HP = sh->HP;
  const size_t n_cap = (size_t)sh->n_cap;
  const bool force_generic = (cfg->flags & NBOS_F_GENERIC_KERNEL) != 0;
  if (batch_mode) {
    h->lds_bytes = 64 + 64 + 128 + (size_t)HP * (32 + 4) + 2 * NGPU * batchk::NCH * 4 + n_cap * 12 + (n_cap + 2) * 2;
    if (h->lds_bytes > (size_t)maxlds) return NBOS_E_LIMIT;
    set_kernel(h, (const void *)batchk::nbos_replay_batch_kernel, "batchk::nbos_replay_batch_kernel%.0u", -1, 0u);
  } else if (closed_loop && cfg->hosts_max <= WAVE && !(cfg->flags & NBOS_F_HOSTS_IN_LDS)) {
    // hosts in registers; 8 bytes per session, 64 staged sessions
    h->lds_bytes = 64 + 64 + 128 + (warm_pool ? (size_t)WAVE * 16 : 0) + n_cap * 8 + WAVE * 4;
    if (h->lds_bytes > (size_t)maxlds) return NBOS_E_LIMIT;
    const int nj = (cfg->hosts_max + 7) / 8;
    const uint32_t policy = cfg->flags & kPolicyFlags;
    if (policy == NBOS_F_MIGRATE && !force_generic) set_reg_closed_kernel<NBOS_F_MIGRATE | NBOS_F_CLOSED_LOOP>(h, nj);
    else set_reg_closed_kernel<kRuntimeClosed>(h, nj);
  } else if (closed_loop) {
    // 12 bytes of record and 4 of timer per session; 64 staged sessions
    h->lds_bytes = 64 + 64 + 128 + 66 * 8 + ldsk::MAIL_WORDS * 4 + (size_t)HP * (32 + 12 + (warm_pool ? 16 : 0)) + n_cap * 12 +
                   (n_cap + 3) / 4 * 16 + WAVE * 4;
    if (h->lds_bytes > (size_t)maxlds) return NBOS_E_LIMIT;
    // instances for the common flag sets, as for the other kernels
    const uint32_t policy = cfg->flags & kPolicyFlags;
    constexpr uint32_t kMigr = NBOS_F_MIGRATE | NBOS_F_CLOSED_LOOP, kMigrOut = kMigr | NBOS_F_SCALE_OUT;
    if (force_generic) set_closed_kernel<kRuntimeClosed>(h);
    else if (policy == NBOS_F_MIGRATE) set_closed_kernel<kMigr>(h);
    else if (policy == (NBOS_F_MIGRATE | NBOS_F_SCALE_OUT)) set_closed_kernel<kMigrOut>(h);
    else set_closed_kernel<kRuntimeClosed>(h);
  } else if (sh->in_regs) {
    h->lds_bytes = 64 + 64 + 128 + (warm_pool ? (size_t)WAVE * 16 : 0) + n_cap * 8 + WAVE * 4;      // + 64 staged sessions
    if (h->lds_bytes > (size_t)maxlds) return NBOS_E_LIMIT;
    const int32_t rc = choose_reg_kernel(h, maxlds);
    if (rc != NBOS_OK) return rc;
  } else {
    // 12 bytes of record and 4 of timer per session; 64 staged sessions
    h->lds_bytes = 64 + 64 + 128 + 66 * 8 + ldsk::MAIL_WORDS * 4 + (size_t)HP * (32 + 12 + (warm_pool ? 16 : 0)) + n_cap * 12 +
                   (n_cap + 3) / 4 * 16 + WAVE * 4;
    if (h->lds_bytes > (size_t)maxlds) return NBOS_E_LIMIT;
    // same idea as for the register kernel; its batches are small (the LDS footprint allows few
    // workgroups per compute unit), so the instance compiled for the flag set is used whenever
    // there is one
    const uint32_t policy = cfg->flags & kPolicyFlags;
    constexpr uint32_t kAllScaling = NBOS_F_MIGRATE | NBOS_F_SCALE_OUT | NBOS_F_SCALE_IN;
    constexpr uint32_t kAutoScaler = NBOS_F_MIGRATE | NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE | NBOS_F_DYNAMIC_SR;
    if (force_generic) set_lds_kernel<kRuntimeFlags>(h);
    else if (policy == kAllScaling) set_lds_kernel<kAllScaling>(h);
    else if (policy == kAutoScaler) set_lds_kernel<kAutoScaler>(h);
    else if (policy == NBOS_F_MIGRATE) set_lds_kernel<NBOS_F_MIGRATE>(h);
    else set_lds_kernel<kRuntimeFlags>(h);
  }
  HIP_TRY(hipFuncSetAttribute(h->kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)h->lds_bytes));
  return NBOS_OK;
}

// device-side validation of the trace contents
int32_t validate_on_device(nbos_replay *h, int64_t slack) {
  const nbos_config *cfg = &h->cfg;
  const nbos_inputs *in = &h->in;
  if (cfg->n_replays == 0) return NBOS_OK;
  uint32_t *d_err = nullptr, h_err = 0;
  if (hipMalloc(&d_err, sizeof(uint32_t)) != hipSuccess) return NBOS_E_NOMEM;
  hipError_t e = hipMemsetAsync(d_err, 0, sizeof(uint32_t), h->stream);
  if (e == hipSuccess) {
    const int32_t t_limit = (int32_t)(0x7FFFFFFELL - slack);
    hipLaunchKernelGGL(nbos_validate_traces, dim3(cfg->n_traces), dim3(256), 0, h->stream, in->ev_offset, in->ev_time_ms,
                       in->ev_dur_ms, in->ev_sess_kind, in->sess_offset, in->sess_gpus, cfg->gpus_per_host,
                       t_limit, d_err);
    hipLaunchKernelGGL(nbos_validate_replays, dim3((cfg->n_replays + 255) / 256), dim3(256), 0, h->stream,
                       in->trace_of_replay, in->cap_milli, cfg->n_replays, cfg->n_traces, d_err);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipMemcpyAsync(&h_err, d_err, sizeof(uint32_t), hipMemcpyDeviceToHost, h->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
  (void)hipFree(d_err);
  if (e != hipSuccess) { note_hip_failure("trace validation", e); return NBOS_E_HIP; }
  return h_err ? NBOS_E_RANGE : NBOS_OK;
}

// result buffers, and what single kernels need beside them
int32_t allocate_buffers(nbos_replay *h, const Shape &sh) {
  const nbos_config *cfg = &h->cfg;
  const nbos_inputs *in = &h->in;
  const size_t n = (size_t)cfg->n_replays;
  if (n == 0) return NBOS_OK;
  if (hipMalloc(&h->d_stats, sizeof(nbos_stats) * n) != hipSuccess) return NBOS_E_NOMEM;
  if (hipMalloc(&h->d_bill, sizeof(nbos_bill) * n) != hipSuccess) return NBOS_E_NOMEM;
  // durations of queued cells whose timers wait outside the sorted registers (open-loop replay kernels)
  const bool queued_durations = !(cfg->flags & (NBOS_F_BATCH_MODE | NBOS_F_CLOSED_LOOP));
  if (queued_durations && hipMalloc(&h->d_ovf, sizeof(int32_t) * n * (size_t)sh.n_cap) != hipSuccess) return NBOS_E_NOMEM;
  if (cfg->flags & NBOS_F_CLOSED_LOOP) {
    // one allocation: chain[total_ev] (two words each), cursor[n_replays][n_cap]; the chains are linked here
    const size_t words = 2 * (size_t)sh.total_ev + n * (size_t)sh.n_cap;
    if (hipMalloc(&h->d_chain, sizeof(int32_t) * (words > 0 ? words : 1)) != hipSuccess) return NBOS_E_NOMEM;
    const size_t chain_lds = (size_t)sh.n_cap * 12;
    HIP_TRY(hipFuncSetAttribute((const void *)ldsk::nbos_closed_chain_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)chain_lds));
    hipLaunchKernelGGL(ldsk::nbos_closed_chain_kernel, dim3(cfg->n_traces), dim3(WAVE), chain_lds, h->stream, in->ev_offset,
                       in->ev_time_ms, in->ev_dur_ms, in->ev_sess_kind, in->sess_offset, (int2 *)h->d_chain);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(h->stream));
  }
  if (cfg->flags & NBOS_F_DECISION_LOG) {
    h->trace_of_replay.resize(n);
    HIP_TRY(hipMemcpyAsync(h->trace_of_replay.data(), in->trace_of_replay, sizeof(int32_t) * n, hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(hipStreamSynchronize(h->stream));
    h->kp.dlog_stride = 3 * (int64_t)sh.max_sess + sh.max_ev + 4096;
    if (hipMalloc(&h->d_log, sizeof(uint64_t) * (size_t)h->kp.dlog_stride * n) != hipSuccess) return NBOS_E_NOMEM;
  }
  return NBOS_OK;
}

// The order in which the launch hands the replays out. Workgroups start in the order of their index (as
// many as fit the chip at once, the others as earlier ones end) and consecutive ones go to different XCDs,
// so a replay's place in that order decides which replays share an XCD and which ones are still running
// when the launch tails off. Longest first: the replays are sorted by the number of events of their trace
// and then by their subscription cap, both descending (on a loaded cluster a higher cap places more
// sessions, and placed sessions are what costs time; on an idle one the cap does not matter). Measured on
// 4,096 replays of 64 hosts with four caps in turn, where every XCD used to get one cap only: 164 -> 104 ms;
// on 16,384 replays of 16 to 24 hosts with random caps: 77 -> 66 ms. Results do not depend on the order:
// every replay writes the records of its own index.
int32_t order_replays(nbos_replay *h) {
  const size_t n = (size_t)h->cfg.n_replays;
  if (n < 2) return NBOS_OK;
  std::vector<int32_t> cap(n), tor(n), order(n);
  HIP_TRY(hipMemcpyAsync(cap.data(), h->in.cap_milli, sizeof(int32_t) * n, hipMemcpyDeviceToHost, h->stream));
  HIP_TRY(hipMemcpyAsync(tor.data(), h->in.trace_of_replay, sizeof(int32_t) * n, hipMemcpyDeviceToHost, h->stream));
  HIP_TRY(hipStreamSynchronize(h->stream));
  for (size_t i = 0; i < n; i++) order[i] = (int32_t)i;
  const std::vector<int64_t> &off = h->ev_off;          // (the validation has checked the trace indices)
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    const int64_t ea = off[tor[a] + 1] - off[tor[a]], eb = off[tor[b] + 1] - off[tor[b]];
    if (ea != eb) return ea > eb;
    return cap[a] > cap[b];
  });
  if (hipMalloc(&h->d_order, sizeof(int32_t) * n) != hipSuccess) return NBOS_E_NOMEM;
  HIP_TRY(hipMemcpyAsync(h->d_order, order.data(), sizeof(int32_t) * n, hipMemcpyHostToDevice, h->stream));
  HIP_TRY(hipStreamSynchronize(h->stream));               // (the host vector goes away)
  return NBOS_OK;
}

// the kernels' parameter block
void fill_params(nbos_replay *h, const Shape &sh) {
  const nbos_config *cfg = &h->cfg;
  const nbos_inputs *in = &h->in;
  KParams &k = h->kp;
  k.ev_offset = in->ev_offset; k.ev_time = in->ev_time_ms; k.ev_dur = in->ev_dur_ms; k.ev_sk = in->ev_sess_kind;
  k.sess_offset = in->sess_offset; k.sess_gpus = in->sess_gpus;
  k.trace_of_replay = in->trace_of_replay; k.cap_milli = in->cap_milli;
  k.stats = h->d_stats; k.dlog = h->d_log; k.ovf_dur = h->d_ovf;       // dlog_stride: set with the log's allocation
  k.order = h->d_order;
  k.n_replays = cfg->n_replays; k.H0 = cfg->hosts_initial; k.Hmax = cfg->hosts_max; k.HP = sh.HP;
  k.G = cfg->gpus_per_host; k.flags = cfg->flags;
  k.migr = cfg->migration_delay_ms; k.boot = cfg->boot_delay_ms; k.retry_iv = cfg->retry_interval_ms;
  k.max_retries = cfg->max_retries;
  k.scale_iv = (cfg->flags & (NBOS_F_SCALE_IN | NBOS_F_AUTOSCALE)) ? cfg->scale_interval_ms : 1;
  k.idle_pct = cfg->scale_in_idle_pct; k.min_hosts = cfg->min_hosts;
  k.f_milli = cfg->autoscale_f_milli; k.buffer = cfg->scaling_buffer_hosts;
  k.batch_delay = cfg->batch_start_delay_ms;
  k.warm_n = (cfg->flags & NBOS_F_WARM_POOL) ? cfg->warm_pool_per_host : 0;
  k.warm_migr = cfg->warm_migration_delay_ms; k.prewarm = cfg->prewarm_delay_ms;
  k.n_cap = sh.n_cap;
  // Event-parallel rounds: on, except for closed loops on clusters of at most 64 hosts, where two
  // cells of a run choose the same host too often for a round to pay (measured: 30 hosts, 110 ms
  // without, 119 ms with). NBOS_F_ROUNDS_OFF / _ON force the choice (comparison runs, tests).
  const bool closed_loop = (cfg->flags & NBOS_F_CLOSED_LOOP) != 0;
  k.batch = (cfg->flags & NBOS_F_ROUNDS_OFF) ? 0 : (cfg->flags & NBOS_F_ROUNDS_ON) ? 1 : (closed_loop && cfg->hosts_max <= WAVE) ? 0 : 1;
  k.cl_chain = (const int2 *)h->d_chain;
  k.cl_cursor = h->d_chain ? h->d_chain + 2 * (size_t)sh.total_ev : nullptr;
}
#undef HIP_TRY
}  // namespace

extern "C" {

const char *nbos_strerror(int32_t status) {
  switch (status) {
    case NBOS_OK: return "ok";
    case NBOS_E_ARG: return "invalid argument";
    case NBOS_E_RANGE: return "invalid trace content";
    case NBOS_E_LIMIT: return "beyond a compiled or device limit";
    case NBOS_E_HIP: return "HIP runtime error";
    case NBOS_E_NOMEM: return "out of memory";
    case NBOS_E_STATE: return "call not valid in this state";
    default: return "unknown status";
  }
}

int32_t nbos_sizeof_stats(void) { return (int32_t)sizeof(nbos_stats); }

const char *nbos_last_error_detail(void) { return g_detail; }

int32_t nbos_replay_create(const nbos_config *cfg_in, const nbos_inputs *in, void *stream, nbos_replay **out) {
  if (out) *out = nullptr;
  if (!cfg_in || !in || !out) return NBOS_E_ARG;
  nbos_config cfg;
  int32_t rc = read_config(cfg_in, &cfg);
  if (rc == NBOS_OK) rc = check_config(&cfg, in);
  if (rc != NBOS_OK) return rc;
  const int64_t slack = time_slack(&cfg);
  if (slack >= 0x7FFFFFFFLL) return NBOS_E_ARG;

  nbos_replay *h = new (std::nothrow) nbos_replay();
  if (!h) return NBOS_E_NOMEM;
  h->cfg = cfg; h->in = *in; h->stream = (hipStream_t)stream;
  h->d_stats = nullptr; h->d_bill = nullptr; h->d_ovf = nullptr; h->d_order = nullptr; h->d_chain = nullptr; h->d_log = nullptr;
  h->kernel = nullptr; h->kernel_name[0] = 0; h->threads = WAVE; h->e0 = nullptr; h->e1 = nullptr; h->ran = false;
  memset(&h->kp, 0, sizeof h->kp);
  Shape sh;
  g_detail[0] = 0;
  rc = open_device(h);
  if (rc == NBOS_OK) rc = read_offsets(h, &sh);
  if (rc == NBOS_OK) rc = choose_kernel(h, &sh);
  if (rc == NBOS_OK) rc = validate_on_device(h, slack);
  if (rc == NBOS_OK) rc = allocate_buffers(h, sh);
  if (rc == NBOS_OK) rc = order_replays(h);
  if (rc != NBOS_OK) { free_handle(h); return rc; }
  fill_params(h, sh);
  *out = h;
  return NBOS_OK;
}

int32_t nbos_replay_run(nbos_replay *h) {
  if (!h) return NBOS_E_ARG;
  if (hipEventRecord(h->e0, h->stream) != hipSuccess) return NBOS_E_HIP;
  if (h->cfg.n_replays > 0) {
    void *args[] = {(void *)&h->kp};
    if (hipLaunchKernel(h->kernel, dim3(h->cfg.n_replays), dim3(h->threads), args, h->lds_bytes, h->stream) != hipSuccess)
      return NBOS_E_HIP;
  }
  if (hipEventRecord(h->e1, h->stream) != hipSuccess) return NBOS_E_HIP;
  h->ran = true;
  return NBOS_OK;
}

int32_t nbos_replay_stats(nbos_replay *h, int32_t first, int32_t count, nbos_stats *host_out) {
  if (!h || first < 0 || count < 0 || (int64_t)first + count > h->cfg.n_replays) return NBOS_E_ARG;
  if (count > 0 && !host_out) return NBOS_E_ARG;
  if (!h->ran) return NBOS_E_STATE;
  if (count > 0 &&
      hipMemcpyAsync(host_out, h->d_stats + first, sizeof(nbos_stats) * (size_t)count, hipMemcpyDeviceToHost,
                     h->stream) != hipSuccess)
    return NBOS_E_HIP;
  if (hipStreamSynchronize(h->stream) != hipSuccess) return NBOS_E_HIP;
  return NBOS_OK;
}

int32_t nbos_replay_billing(nbos_replay *h, const nbos_billing_params *bp, int32_t first, int32_t count,
                            nbos_bill *host_out) {
  if (!h || !bp || first < 0 || count < 0 || (int64_t)first + count > h->cfg.n_replays) return NBOS_E_ARG;
  if (count > 0 && !host_out) return NBOS_E_ARG;
  if (bp->price_micro_per_host_hour < 0 || bp->price_micro_per_host_hour > 1000000000LL) return NBOS_E_ARG;
  if (bp->markup_pct < 0 || bp->markup_pct > 1000 || bp->standby_permille < 0 || bp->standby_permille > 1000)
    return NBOS_E_ARG;
  if (!h->ran) return NBOS_E_STATE;
  if (count > 0) {
    hipLaunchKernelGGL(nbos_billing_kernel, dim3((count + 255) / 256), dim3(256), 0, h->stream, h->d_stats, first,
                       count, h->cfg.gpus_per_host, bp->price_micro_per_host_hour, bp->markup_pct,
                       bp->standby_permille, h->d_bill);
    if (hipGetLastError() != hipSuccess) return NBOS_E_HIP;
    if (hipMemcpyAsync(host_out, h->d_bill, sizeof(nbos_bill) * (size_t)count, hipMemcpyDeviceToHost, h->stream) !=
        hipSuccess)
      return NBOS_E_HIP;
  }
  if (hipStreamSynchronize(h->stream) != hipSuccess) return NBOS_E_HIP;
  return NBOS_OK;
}

int64_t nbos_replay_decisions(nbos_replay *h, int32_t replay, uint64_t *host_out, int64_t cap) {
  if (!h || replay < 0 || replay >= h->cfg.n_replays || cap < 0 || (cap > 0 && !host_out)) return NBOS_E_ARG;
  if (!(h->cfg.flags & NBOS_F_DECISION_LOG) || !h->ran) return NBOS_E_STATE;
  nbos_stats st;
  if (hipMemcpyAsync(&st, h->d_stats + replay, sizeof st, hipMemcpyDeviceToHost, h->stream) != hipSuccess) return NBOS_E_HIP;
  if (hipStreamSynchronize(h->stream) != hipSuccess) return NBOS_E_HIP;
  int64_t logged = st.n_decisions < (uint64_t)h->kp.dlog_stride ? (int64_t)st.n_decisions : h->kp.dlog_stride;
  int64_t n = logged < cap ? logged : cap;
  if (n > 0) {
    if (hipMemcpyAsync(host_out, h->d_log + (int64_t)replay * h->kp.dlog_stride, sizeof(uint64_t) * (size_t)n,
                       hipMemcpyDeviceToHost, h->stream) != hipSuccess) return NBOS_E_HIP;
    if (hipStreamSynchronize(h->stream) != hipSuccess) return NBOS_E_HIP;
  }
  return logged;
}

int32_t nbos_replay_last_kernel_ms(nbos_replay *h, float *ms_out) {
  if (!h || !ms_out) return NBOS_E_ARG;
  if (!h->ran) return NBOS_E_STATE;
  if (hipEventSynchronize(h->e1) != hipSuccess) return NBOS_E_HIP;
  if (hipEventElapsedTime(ms_out, h->e0, h->e1) != hipSuccess) return NBOS_E_HIP;
  return NBOS_OK;
}

int32_t nbos_replay_launch_info(nbos_replay *h, int32_t *lds_bytes, int32_t *threads_per_group, int32_t *groups) {
  if (!h) return NBOS_E_ARG;
  if (lds_bytes) *lds_bytes = (int32_t)h->lds_bytes;
  if (threads_per_group) *threads_per_group = h->threads;
  if (groups) *groups = h->cfg.n_replays;
  return NBOS_OK;
}

int32_t nbos_replay_run_static(const nbos_config *cfg_in, const nbos_inputs *in, int32_t max_sessions_per_trace,
                               void *stream, nbos_stats *device_stats_out) {
  if (!cfg_in || !in) return NBOS_E_ARG;
  nbos_config cfg;
  int32_t rc = read_config(cfg_in, &cfg);
  if (rc == NBOS_OK) rc = check_config(&cfg, in);
  if (rc != NBOS_OK) return rc;
  const int64_t slack = time_slack(&cfg);
  if (slack >= 0x7FFFFFFFLL) return NBOS_E_ARG;
  if (cfg.n_replays == 0) return NBOS_OK;
  if (!device_stats_out || max_sessions_per_trace < 0 || max_sessions_per_trace > NBOS_MAX_SESSIONS) return NBOS_E_ARG;
  if (!in->ev_time_ms || !in->ev_dur_ms || !in->ev_sess_kind || !in->sess_gpus) return NBOS_E_ARG;
  // only the kernel with the hosts in registers runs here, without a log, as an open loop
  if (cfg.flags & (NBOS_F_DECISION_LOG | NBOS_F_HOSTS_IN_LDS | NBOS_F_BATCH_MODE | NBOS_F_CLOSED_LOOP)) return NBOS_E_ARG;
  if (cfg.hosts_max > WAVE) return NBOS_E_LIMIT;
  const size_t n_cap = max_sessions_per_trace > 0 ? (size_t)max_sessions_per_trace : 1;
  if ((size_t)cfg.n_replays * n_cap > kScratchWords - kScratchHead) return NBOS_E_LIMIT;

  // this GPU's copy of the scratch array: looked up once per device, with that device current
  static std::mutex mu;
  static int32_t *scratch_of[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return NBOS_E_HIP;
  if (dev < 0 || dev >= 64) return NBOS_E_LIMIT;
  int32_t *base = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!scratch_of[dev]) {
      void *ptr = nullptr;
      const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !ptr) { note_hip_failure("hipGetSymbolAddress(scratch)", e); return NBOS_E_HIP; }
      scratch_of[dev] = (int32_t *)ptr;
    }
    base = scratch_of[dev];
  }

  nbos_replay tmp{};                      // never leaves this call; its vectors stay empty
  tmp.cfg = cfg; tmp.in = *in; tmp.stream = (hipStream_t)stream; tmp.device = dev; tmp.threads = WAVE;
  const bool warm_pool = (cfg.flags & NBOS_F_WARM_POOL) != 0;
  tmp.lds_bytes = 64 + 64 + 128 + (warm_pool ? (size_t)WAVE * 16 : 0) + n_cap * 8 + WAVE * 4;
  int maxlds = 0;
  if (hipDeviceGetAttribute(&maxlds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return NBOS_E_HIP;
  if (tmp.lds_bytes > (size_t)maxlds) return NBOS_E_LIMIT;
  rc = choose_reg_kernel(&tmp, maxlds);
  if (rc != NBOS_OK) return rc;
  if (hipFuncSetAttribute(tmp.kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)tmp.lds_bytes) != hipSuccess)
    return NBOS_E_HIP;
  Shape sh;
  sh.HP = WAVE; sh.n_cap = (int)n_cap; sh.in_regs = true;
  tmp.d_stats = device_stats_out;
  tmp.d_ovf = base + kScratchHead;
  fill_params(&tmp, sh);
  uint32_t *err = (uint32_t *)base;
  tmp.kp.trace_err = err;

  hipStream_t st = tmp.stream;
  const int32_t t_limit = (int32_t)(0x7FFFFFFELL - slack);
  hipLaunchKernelGGL(nbos_clear_word, dim3(1), dim3(1), 0, st, err);
  hipLaunchKernelGGL(nbos_validate_offsets, dim3((cfg.n_traces + 256) / 256), dim3(256), 0, st, in->ev_offset,
                     in->sess_offset, cfg.n_traces, err);
  hipLaunchKernelGGL(nbos_validate_replays, dim3((cfg.n_replays + 255) / 256), dim3(256), 0, st, in->trace_of_replay,
                     in->cap_milli, cfg.n_replays, cfg.n_traces, err);
  hipLaunchKernelGGL(nbos_validate_traces_checked, dim3(cfg.n_traces), dim3(256), 0, st, in->ev_offset, in->ev_time_ms,
                     in->ev_dur_ms, in->ev_sess_kind, in->sess_offset, in->sess_gpus, cfg.gpus_per_host, t_limit, err);
  if (hipGetLastError() != hipSuccess) return NBOS_E_HIP;
  void *args[] = {(void *)&tmp.kp};
  if (hipLaunchKernel(tmp.kernel, dim3(cfg.n_replays), dim3(WAVE), args, tmp.lds_bytes, st) != hipSuccess) return NBOS_E_HIP;
  return NBOS_OK;
}

#ifdef NBOS_PATH_PROFILE
// Diagnostic build only (not declared in nbos.h): the path profile of the last launch of an open-loop replay
// kernel, host_out[replay][0 = clocks, 1 = counts][category], PC_N categories, the first `replays` replays.
int32_t nbos_path_profile_read(unsigned long long *host_out, int32_t replays, int32_t *categories) {
  if (categories) *categories = PC_N;
  if (!host_out || replays < 0 || replays > PATH_PROFILE_REPLAYS) return NBOS_E_ARG;
  if (hipDeviceSynchronize() != hipSuccess) return NBOS_E_HIP;
  return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_path_profile), sizeof(unsigned long long) * 2 * PC_N * (size_t)replays, 0,
                             hipMemcpyDeviceToHost) == hipSuccess ? NBOS_OK : NBOS_E_HIP;
}
#endif

const char *nbos_replay_kernel_name(nbos_replay *h) { return h ? h->kernel_name : ""; }

int32_t nbos_chain_floor_ns(void *stream, int32_t iters, float *ns_out) {
  if (!ns_out || iters < 1 || iters > (1 << 24)) return NBOS_E_ARG;
  hipStream_t st = (hipStream_t)stream;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return NBOS_E_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return NBOS_E_HIP;
  uint32_t *sink = nullptr;
  if (hipMalloc(&sink, sizeof(uint32_t) * (size_t)cus) != hipSuccess) return NBOS_E_NOMEM;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  float ms = 0.f;
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
  for (int pass = 0; pass < 2 && ok; pass++) {          // the first pass warms the clocks up
    ok = hipEventRecord(e0, st) == hipSuccess;
    if (ok) {
      hipLaunchKernelGGL(nbos_chain_floor_kernel, dim3(cus), dim3(WAVE), 0, st, iters, sink);
      ok = hipGetLastError() == hipSuccess && hipEventRecord(e1, st) == hipSuccess &&
           hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    }
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  if (!ok) return NBOS_E_HIP;
  *ns_out = ms * 1e6f / (float)iters;
  return NBOS_OK;
}

void nbos_replay_destroy(nbos_replay *h) {
  if (!h) return;
  (void)hipStreamSynchronize(h->stream);
  free_handle(h);
}

}  // extern "C"
