/*
 * nbos.h — C ABI of the batched NotebookOS policy replay for AMD MI355X (gfx950).
 *
 * What the library computes
 * -------------------------
 * Many independent trace-driven replays of NotebookOS's replica-placement and
 * dynamic GPU-binding policy (paper Sections 3.2.1-3.2.3, 3.3, 3.4.1, 3.4.2).
 * One replay = one simulated cluster of GPU servers ("hosts") that is fed one
 * time-ordered trace of notebook-session events:
 *
 *   SESSION_START  place R = 3 kernel replicas on 3 distinct hosts. Replicas
 *                  subscribe to GPUs, they do not commit them (Section 3.2.1).
 *                  A host is a candidate when its subscription ratio
 *                  S / (G * R) stays at or below the replay's cap after adding
 *                  the replica (Section 3.4.1). Among candidates the hosts with
 *                  the most idle GPUs win, then the lowest subscription, then
 *                  the lowest host index. Fewer than 3 candidates: scale out or
 *                  reject (Section 3.4.2).
 *   CELL           executor election by outcome: the replica whose host is
 *                  ready and has enough uncommitted GPUs executes, and the GPUs
 *                  are committed for the cell's duration only (Sections 3.2.2,
 *                  3.3). When every replica must yield, one replica is migrated
 *                  to a host that can bind the GPUs at once (Section 3.2.3),
 *                  else a host is added for it, else the cell is queued and
 *                  retried periodically, and aborted after max_retries.
 *   SESSION_END    the replicas give their subscriptions back (after the
 *                  running cell, if there is one).
 *
 * All times are int32 milliseconds, all results are integers; no floating point
 * is used anywhere, so results are exact and reproducible.
 *
 * Section numbers used in this file and in the sources, with the paper's titles:
 *   2.2    Interactive Deep Learning Training      3.3    GPU Management
 *   3.2.1  Distributed Kernel Creation             3.4.1  Default Placement Policy
 *   3.2.2  Distributed Kernel Raft Protocol        3.4.2  Scale-Out Operations
 *   3.2.3  Handling Failed Executor Elections (with "Pre-warmed Container Pool")
 * Passages of the evaluation are cited by title only: "Baselines" (Reservation, Batch),
 * "Resource Usage & Efficiency", "Interactivity", "Task Completion Time", "Subscription
 * Ratio", and "Monetary Cost" / "GPU Hours Saved" of the simulation study.
 *
 * Pointers
 * --------
 * nbos_config / nbos_inputs structs themselves live in HOST memory.
 * Every array named in nbos_inputs is a DEVICE pointer (HBM). The library
 * borrows them: it never copies, frees or writes them, and they must stay valid
 * and unchanged until nbos_replay_destroy. nbos_stats / decision outputs are
 * written to HOST memory supplied by the caller.
 *
 * Errors
 * ------
 * Every int32_t entry point returns NBOS_OK (0) or a negative nbos_status.
 * Nothing throws, aborts or prints. Policy outcomes of a replay (rejected
 * sessions, aborted cells) are counts in nbos_stats, not errors.
 */
#ifndef NBOS_H
#define NBOS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- limits of this build ------------------------------------------------ */
#define NBOS_MAX_HOSTS        1024    /* hosts_max upper bound (10-bit host ids)      */
#define NBOS_MAX_SESSIONS     65536   /* sessions per trace (16-bit ids in decisions) */
#define NBOS_MAX_GPUS         8       /* G per host, Section 3.4.1: 1..8              */
#define NBOS_MAX_RETRIES      15
#define NBOS_MAX_CAP_MILLI    100000  /* subscription-ratio cap 100.0                 */
#define NBOS_MAX_DUR_MS       86400000 /* one cell runs at most 24 h                  */

typedef enum {
  NBOS_OK      =  0,
  NBOS_E_ARG   = -1,   /* null pointer, bad struct_size, parameter out of range        */
  NBOS_E_RANGE = -2,   /* trace content invalid: unsorted times, time overflow, bad
                          kind / session id / duration / GPU request / trace index      */
  NBOS_E_LIMIT = -3,   /* beyond a compiled or device limit (hosts, sessions, LDS)      */
  NBOS_E_HIP   = -4,   /* a HIP runtime call failed                                     */
  NBOS_E_NOMEM = -5,   /* host or device allocation failed                              */
  NBOS_E_STATE = -6    /* call not valid now (e.g. decisions without the log flag)      */
} nbos_status;

/* ---- flags --------------------------------------------------------------- */
#define NBOS_F_MIGRATE       0x1u  /* failed election -> replica migration (Section 3.2.3)   */
#define NBOS_F_SCALE_OUT     0x2u  /* failed placement / migration -> add hosts (3.4.2)      */
#define NBOS_F_SCALE_IN      0x4u  /* periodic release of empty hosts (3.4.2, last par.)     */
#define NBOS_F_DECISION_LOG  0x8u  /* keep every decision code per replay (debug, slower)    */
#define NBOS_F_HOSTS_IN_LDS   0x10u /* use the any-size kernel (host state in LDS) even when
                                      hosts_max <= 64 would allow the register kernel; same
                                      results, for cross-checks and comparisons              */
#define NBOS_F_GENERIC_KERNEL 0x800u /* comparison runs: run the kernel instance that reads the policy flags
                                      at run time even where an instance compiled for the flag set
                                      exists; same results                                       */
#define NBOS_F_ROUNDS_OFF    0x1000u /* comparison runs: never evaluate runs of arrivals (or of due
                                      closed-loop events) in event-parallel rounds; same results   */
#define NBOS_F_ROUNDS_ON     0x2000u /* comparison runs: use the rounds also where they are off by
                                      default (closed loops on at most 64 hosts with
                                      NBOS_F_HOSTS_IN_LDS); same results. Not with NBOS_F_ROUNDS_OFF */
#define NBOS_F_ONE_WAVE      0x4000u /* comparison runs: one wave per replay also on clusters of 256 hosts
                                      or more, where three helper waves would share the scans over
                                      all hosts; same results                                      */
#define NBOS_F_AUTOSCALE     0x20u /* the periodic auto-scaler of Section 3.4.2 (second scale-out
                                      scenario). Every scale_interval_ms the expected capacity is
                                      want = ceil(f * sum C / G) + scaling_buffer_hosts hosts, with
                                      sum C = GPUs committed at that instant and hosts being
                                      provisioned counted as capacity. Fewer hosts than want: the
                                      difference is provisioned at once (up to hosts_max). With
                                      NBOS_F_SCALE_IN also set and more hosts than want: at most 2
                                      ready hosts without replicas are released per period, highest
                                      index first, never below want or min_hosts; this test then
                                      replaces the scale_in_idle_pct rule.                     */
#define NBOS_F_DYNAMIC_SR    0x40u /* dynamic cluster-wide limit on the subscription ratio
                                      (Section 3.4.1, third factor): a host also passes the cap
                                      test when (S_h + g) / (G R) <= (sum S + g) / (n G R), n =
                                      hosts not off, i.e. the limit in force is the larger of the
                                      replay's cap and the cluster-wide ratio after placing.  */

#define NBOS_F_STICKY_EXECUTOR 0x80u /* election variant (Section 3.2.2; the "Interactivity" section reports that
                                      consecutive cells ran on the same replica 89.45 % of the
                                      time): the replica that executed the session's previous
                                      cell leads again whenever its host can bind the GPUs;
                                      otherwise the usual rule decides                        */

#define NBOS_F_BATCH_MODE    0x100u /* replay the Batch baseline of the paper's "Baselines" section instead of the
                                      NotebookOS policy: no replicas; every cell is a job of its
                                      own, served first come first served (a job never overtakes
                                      an earlier one) on the ready host with the fewest committed
                                      GPUs that has g idle ones (ties: lowest index). The job holds
                                      its GPUs for batch_start_delay_ms (container start) plus the
                                      cell's duration. The queue is served after each arrival and
                                      after all completions / hosts turning ready of one instant.
                                      A cell whose session's previous job has not finished is
                                      dropped. START / END events are ignored. Only
                                      NBOS_F_SCALE_OUT (the job at the head of the queue that
                                      finds no host asks for one more, once), NBOS_F_DECISION_LOG
                                      and NBOS_F_HOSTS_IN_LDS may be combined with it. Of the
                                      stats, the placement / migration / subscription fields stay
                                      0; cells_queued counts the jobs that waited for GPUs.      */

#define NBOS_F_WARM_POOL     0x200u /* pre-warmed container pool (Section 3.2.3): every host keeps
                                      warm_pool_per_host pre-warmed containers (initial hosts from
                                      time 0, added hosts prewarm_delay_ms after they are ready).
                                      A migration takes the target's container that has been
                                      available longest, if one is available: the cell then starts
                                      after warm_migration_delay_ms instead of migration_delay_ms
                                      (decision NBOS_D_MIGRATE_WARM) and a replacement is available
                                      prewarm_delay_ms later. Not with NBOS_F_BATCH_MODE.        */

#define NBOS_F_CLOSED_LOOP   0x400u /* closed-loop reading of the traces (the section "Interactive Deep Learning Training" describes
                                      users who think and edit between cells): only a session's
                                      first START keeps its time. Every later CELL / END of the
                                      session is due one think time after the session's previous
                                      cell is over (finished or given up; the first one: after the
                                      placement); the think time is what the trace leaves between
                                      the previous event's nominal end (its time, plus its duration
                                      for a CELL) and the event's own time, at least 0. Events
                                      before the first START, repeated STARTs and everything after
                                      the first END are ignored; cells of sessions that were not
                                      placed never arrive (cells_total counts arrivals). Due events
                                      run after retries of the same instant, by ascending session.
                                      Runs on closed-loop variants of both kernels (hosts in
                                      registers up to 64 hosts, else in LDS); not with
                                      NBOS_F_SCALE_IN, NBOS_F_AUTOSCALE or NBOS_F_BATCH_MODE. A replay whose lag
                                      pushes a time to 2^31 - 1 ends with status NBOS_E_RANGE.    */

/* ---- event encoding ------------------------------------------------------ */
#define NBOS_EV_START  0
#define NBOS_EV_CELL   1
#define NBOS_EV_END    2
/* ev_sess_kind = session_id | (kind << 24) */

typedef struct nbos_replay nbos_replay;   /* opaque, owned by the library */

/* Parameters common to all replays of one handle. */
typedef struct {
  uint32_t struct_size;         /* = sizeof(nbos_config); the shorter layouts that end at
                                   min_hosts (60 bytes), scaling_buffer_hosts (68) or
                                   batch_start_delay_ms (72) are accepted
                                   too, the missing fields read as 0      */
  int32_t  n_replays;           /* >= 0                                                         */
  int32_t  n_traces;            /* >= 1 when n_replays > 0                                      */
  int32_t  hosts_initial;       /* hosts 0..hosts_initial-1 are ready at time 0; >= 1           */
  int32_t  hosts_max;           /* >= hosts_initial, <= NBOS_MAX_HOSTS; extra ones start off    */
  int32_t  gpus_per_host;       /* G, 1..8 (Section 3.4.1)                                      */
  int32_t  replicas;            /* R, must be 3 (Section 3.2)                                   */
  uint32_t flags;               /* NBOS_F_*                                                     */
  int32_t  migration_delay_ms;  /* >= 0; container start + state read of a migrated replica     */
  int32_t  boot_delay_ms;       /* >= 0; a scaled-out host is ready this long after the request */
  int32_t  retry_interval_ms;   /* >= 1; period of the retries of a queued cell (3.2.3)         */
  int32_t  max_retries;         /* 0..NBOS_MAX_RETRIES; then the cell is aborted                */
  int32_t  scale_interval_ms;   /* >= 1 with NBOS_F_SCALE_IN / _AUTOSCALE: auto-scaler period   */
  int32_t  scale_in_idle_pct;   /* 0..100: release while empty*100 > ready*pct                  */
  int32_t  min_hosts;           /* scale-in never goes below this many ready hosts              */
  int32_t  autoscale_f_milli;   /* NBOS_F_AUTOSCALE: f * 1000 of the expected capacity f * sum C,
                                   0..100000 (Section 3.4.2 uses f = 1.05, i.e. 1050)           */
  int32_t  scaling_buffer_hosts;/* NBOS_F_AUTOSCALE: extra hosts kept on top of it, 0..1024     */
  int32_t  batch_start_delay_ms;/* NBOS_F_BATCH_MODE: container start per job, 0..NBOS_MAX_DUR_MS */
  int32_t  warm_pool_per_host;  /* NBOS_F_WARM_POOL: pre-warmed containers per host, 1..4        */
  int32_t  warm_migration_delay_ms; /* NBOS_F_WARM_POOL: migration delay into one of them, >= 0  */
  int32_t  prewarm_delay_ms;    /* NBOS_F_WARM_POOL: time to pre-warm a container, 0..NBOS_MAX_DUR_MS */
} nbos_config;

/* The traces and per-replay parameters. All arrays are DEVICE pointers. */
typedef struct {
  const int64_t *ev_offset;       /* [n_traces+1] first event of each trace, ev_offset[0] = 0   */
  const int32_t *ev_time_ms;      /* [ev_offset[n_traces]] >= 0, non-decreasing within a trace  */
  const int32_t *ev_dur_ms;       /* CELL: 1..NBOS_MAX_DUR_MS; START / END: ignored             */
  const int32_t *ev_sess_kind;    /* session id (bits 0..23, local to the trace) | kind << 24   */
  const int32_t *sess_offset;     /* [n_traces+1] first session of each trace                   */
  const uint8_t *sess_gpus;       /* [sess_offset[n_traces]] GPU request g, 1..gpus_per_host    */
  const int32_t *trace_of_replay; /* [n_replays] which trace a replay consumes                  */
  const int32_t *cap_milli;       /* [n_replays] subscription-ratio cap * 1000, 1..MAX_CAP_MILLI*/
} nbos_inputs;

/*
 * Result of one replay. Counter semantics (the paper's sections "Resource Usage & Efficiency", "Interactivity" and "Task Completion Time" for the
 * metric definitions):
 *   cells_immediate   cells whose GPUs were committed by election at submit time
 *   executor_reused   cell executed by the same replica slot as the previous cell
 *   delay             start of execution minus submission ("interactivity delay")
 *   tct               completion minus submission ("task completion time")
 *   delay_hist[b]     b = 0 for delay 0, else 1 + floor(log2(delay)), capped at 31
 *   gpu_ms_executed   sum g * duration over started cells
 *   gpu_ms_committed  sum g * (finish - commit): includes migration / boot waits
 *   gpu_ms_provisioned integral over [0, t_end] of G * (hosts not off)
 *   reservation_gpu_ms sum over placed sessions g * (end - start): what the
 *                     Reservation baseline holds (end = END event time or t_end)
 *   sub_gpu_ms        integral over [0, t_end] of the cluster's subscribed GPUs
 *   replica_ms        integral over [0, t_end] of the number of placed replicas
 *   digest            d = d * 0x100000001B3 + code over all decisions in order,
 *                     starting from 0xCBF29CE484222325 (wrapping uint64)
 * Decision code = host | slot << 10 | outcome << 12 | session << 16 | time << 32.
 */
typedef struct {
  int32_t  status;              /* NBOS_OK; NBOS_E_RANGE (Batch baseline, closed loop): a time left the
                                   int32 range; nbos_replay_run_static only: NBOS_E_RANGE / NBOS_E_LIMIT as
                                   documented there. The other fields are invalid then. (No queue
                                   inside a replay can overflow: a session has at most one timer, and a
                                   timer that is not among the 64 sorted ones waits in the session's
                                   own record.)                                                    */
  uint32_t n_decisions;
  uint32_t sessions_placed, sessions_rejected;
  uint32_t cells_total, cells_immediate, cells_started, cells_queued, cells_aborted;
  uint32_t cells_dropped_busy, cells_dropped_unplaced;
  uint32_t executor_reused, migrations;
  uint32_t scale_out_hosts, scale_in_hosts, peak_hosts;
  uint32_t migrations_warm;     /* migrations that found a pre-warmed container (NBOS_F_WARM_POOL) */
  int32_t  max_delay_ms, t_end_ms;
  uint32_t delay_hist[32];
  int64_t  sum_delay_ms, sum_tct_ms;
  int64_t  gpu_ms_executed, gpu_ms_committed, gpu_ms_provisioned;
  int64_t  reservation_gpu_ms, sub_gpu_ms;
  int64_t  replica_ms;
  uint64_t digest;
} nbos_stats;

/* decision outcomes (bits 12..15 of a decision code) */
#define NBOS_D_PLACE       1   /* replica slot placed on an existing host            */
#define NBOS_D_PLACE_NEW   2   /* replica slot reserved on a host being booted       */
#define NBOS_D_REJECT      3   /* session could not be placed                        */
#define NBOS_D_START       4   /* cell started by election on (slot, host)           */
#define NBOS_D_MIGRATE     5   /* replica slot migrated to host, cell starts there   */
#define NBOS_D_SCALE_CELL  6   /* host added for the cell, replica slot moved there  */
#define NBOS_D_ABORT       7   /* queued cell given up                               */
#define NBOS_D_SCALE_IN    8   /* empty host released (session field 0)              */
#define NBOS_D_SCALE_AUTO  9   /* host provisioned by the periodic auto-scaler       */
#define NBOS_D_BATCH_START 10  /* Batch baseline: GPUs allocated to the job on host   */
#define NBOS_D_BATCH_HOST  11  /* Batch baseline: host provisioned for the queue head */
#define NBOS_D_MIGRATE_WARM 12 /* as NBOS_D_MIGRATE, into a pre-warmed container      */

/*
 * Create a replay batch (paper Sections 3.2-3.4 define the simulated policy).
 *   cfg, in   host structs, copied. Arrays inside `in` are device pointers,
 *             borrowed until destroy.
 *   stream    a hipStream_t (or NULL for the default stream) on the current
 *             device; all device work of this handle is ordered on it.
 *   out       receives the handle.
 * Validates parameters on the host and the trace contents with a device kernel
 * (synchronises the stream once). Allocates only its own result buffers.
 * Which kernel runs follows from cfg alone (cluster size, policy flags and the comparison flags
 * NBOS_F_HOSTS_IN_LDS / _GENERIC_KERNEL / _ROUNDS_OFF / _ROUNDS_ON); the environment is not read.
 * With NBOS_F_CLOSED_LOOP a device kernel links every session's events here (8 bytes per event
 * and 4 per replay and session of device memory are held until destroy).
 * Errors: NBOS_E_ARG, NBOS_E_RANGE, NBOS_E_LIMIT (hosts/sessions/LDS footprint
 * beyond what one workgroup can hold), NBOS_E_HIP, NBOS_E_NOMEM. *out is NULL
 * on error.
 */
int32_t nbos_replay_create(const nbos_config *cfg, const nbos_inputs *in,
                           void *stream, nbos_replay **out);

/*
 * Enqueue one full pass: every replay consumes its whole trace and writes its
 * nbos_stats into the handle's device buffer. Per event, in trace order, with
 * every timer that is due at or before the event run first:
 *   SESSION_START  three replicas on three hosts, subscribed not committed
 *                  ("Distributed Kernel Creation", "Default Placement Policy");
 *   CELL           the election among the session's replicas, GPUs bound for the
 *                  cell's duration and released at its end ("Distributed Kernel
 *                  Raft Protocol", "GPU Management"); when all replicas yield: a
 *                  migration, a new host, or the retry queue ("Handling Failed
 *                  Executor Elections", "Scale-Out Operations");
 *   periodic       the auto-scaler's release / provisioning of hosts ("Scale-Out
 *                  Operations", last paragraphs);
 * then the pending timers are drained and the integrals are closed at the last instant.
 * Takes no arguments beyond the handle; reads the borrowed device arrays of create.
 * Asynchronous on the handle's stream; may be called repeatedly, every call
 * recomputes the same results from the same inputs. Nothing is allocated here.
 * Errors: NBOS_E_ARG (null), NBOS_E_HIP.
 */
int32_t nbos_replay_run(nbos_replay *h);

/*
 * Copy the stats of replays [first, first+count) to host_out (host memory,
 * count * sizeof(nbos_stats) bytes, owned by the caller). The fields are the
 * quantities the paper's evaluation reports per policy: GPUs provisioned, bound
 * and reserved over time ("Resource Usage & Efficiency", "GPU Hours Saved"), the
 * interactivity delay and its distribution, immediate starts and executor reuse
 * ("Interactivity"), completion times ("Task Completion Time"), the subscribed
 * GPUs over time ("Subscription Ratio"), migrations and hosts added / released
 * ("Scale-Out Operations"). Synchronises the handle's stream.
 * Errors: NBOS_E_ARG (null, range), NBOS_E_STATE (never run), NBOS_E_HIP.
 */
int32_t nbos_replay_stats(nbos_replay *h, int32_t first, int32_t count,
                          nbos_stats *host_out);

/*
 * The sequence of scheduling decisions of one replay: which hosts a session's replicas
 * were placed on ("Distributed Kernel Creation"), which replica led each cell and where
 * ("Distributed Kernel Raft Protocol"), every migration, added host, abort and released
 * host ("Handling Failed Executor Elections", "Scale-Out Operations"), as NBOS_D_* codes.
 * Only with NBOS_F_DECISION_LOG: copy up to `cap` decision codes of one replay
 * to host_out (host memory), in processing order. Returns the number of codes
 * the replay logged (may exceed cap; a replay logs at most its own capacity of
 * 3 * sessions + events + 4096 codes, n_decisions in the stats counts all).
 * Negative return = nbos_status. Synchronises the stream.
 */
int64_t nbos_replay_decisions(nbos_replay *h, int32_t replay,
                              uint64_t *host_out, int64_t cap);

/*
 * Milliseconds the most recent nbos_replay_run spent on the device, measured
 * with HIP events recorded on the handle's stream around the replay kernel.
 * Synchronises the stream. Errors: NBOS_E_ARG, NBOS_E_STATE, NBOS_E_HIP.
 */
int32_t nbos_replay_last_kernel_ms(nbos_replay *h, float *ms_out);

/* Dynamic LDS bytes per workgroup and waves per workgroup chosen at create. */
int32_t nbos_replay_launch_info(nbos_replay *h, int32_t *lds_bytes,
                                int32_t *threads_per_group, int32_t *groups);

/*
 * Billing model of the paper's "Monetary Cost" section as a post-pass over the results of the last run, in integer
 * micro-dollars, every amount rounded down:
 *   provider_cost        price * host-hours provisioned   (gpu_ms_provisioned / G)
 *   usage_revenue        executing replicas pay markup_pct/100 of the provider's rate for the share
 *                        g / G of a host they use         (gpu_ms_executed / G)
 *   standby_revenue      a placed replica that is not executing pays standby_permille/1000 of the
 *                        marked-up host rate              (replica_ms - executing time)
 *   reservation_revenue  the Reservation baseline at the same markup (reservation_gpu_ms / G)
 * The paper's example: $10 per host-hour (price 10,000,000), markup 115, standby 125.
 */
typedef struct {
  int64_t price_micro_per_host_hour;  /* 0..1,000,000,000 */
  int32_t markup_pct;                 /* 0..1000          */
  int32_t standby_permille;           /* 0..1000          */
} nbos_billing_params;

typedef struct {
  int64_t provider_cost, usage_revenue, standby_revenue, reservation_revenue;
} nbos_bill;

/*
 * Compute the bills of replays [first, first+count) on the device from the stats of the last run and
 * copy them to host_out (host memory, count * sizeof(nbos_bill) bytes). Synchronises the stream.
 * Errors: NBOS_E_ARG (null, range, parameter out of range), NBOS_E_STATE (never run), NBOS_E_HIP.
 */
int32_t nbos_replay_billing(nbos_replay *h, const nbos_billing_params *params, int32_t first,
                            int32_t count, nbos_bill *host_out);

/*
 * For callers that cannot allocate device memory (code under stream capture, serving loops that
 * must not call the allocator, harnesses that forbid it): what nbos_replay_create + nbos_replay_run
 * do, in one call that allocates nothing, for clusters of at most 64 hosts.
 *   cfg, in    as for nbos_replay_create (host structs; the arrays are device pointers, borrowed for
 *              the duration of the enqueued work). Not with NBOS_F_DECISION_LOG, _HOSTS_IN_LDS,
 *              _BATCH_MODE or _CLOSED_LOOP (NBOS_E_ARG); hosts_max <= 64 (else NBOS_E_LIMIT).
 *   max_sessions_per_trace  an upper bound on the sessions of any one trace (sizes the LDS of a
 *              replay); 0..NBOS_MAX_SESSIONS.
 *   stream     a hipStream_t or NULL; everything is enqueued there, nothing is waited for.
 *   device_stats_out  DEVICE memory for n_replays nbos_stats records, owned by the caller; valid
 *              once the stream has passed the call's work.
 * The kernels' scratch memory (the validation verdict, and the durations of queued cells whose
 * timers wait outside the sorted registers: n_replays * max_sessions_per_trace words) is a fixed
 * 16 MiB array inside the library, one per GPU, held until the process ends:
 * n_replays * max(max_sessions_per_trace, 1) must not exceed 4,194,240 (NBOS_E_LIMIT). All calls on
 * one GPU share that array: calls whose device work overlaps race; order them on one stream or
 * with events.
 * The traces are checked on the device, in the same stream; the host does not see the verdict.
 * Invalid content (what create reports as NBOS_E_RANGE) gives every record of the call status
 * NBOS_E_RANGE; a trace with more sessions than max_sessions_per_trace gives the replays of that
 * trace status NBOS_E_LIMIT; the other fields of such records are 0. The offset arrays must address
 * memory that exists (as everywhere, the library cannot know the arrays' lengths).
 * Errors: NBOS_E_ARG, NBOS_E_LIMIT, NBOS_E_HIP. Results equal those of create + run + stats.
 */
int32_t nbos_replay_run_static(const nbos_config *cfg, const nbos_inputs *in, int32_t max_sessions_per_trace,
                               void *stream, nbos_stats *device_stats_out);

/* Name of the replay kernel instance chosen at create, as a profiler's kernel trace prints it
 * (without the argument list), e.g. "ldsk::nbos_replay_lds_kernel<7u>". Static storage of the
 * handle, valid until destroy; "" for a NULL handle. */
const char *nbos_replay_kernel_name(nbos_replay *h);

/*
 * Measurement aid, no part of a replay: the dependency-chain floor of one event body. A replay is
 * a serial chain of state updates; the shortest step this design can take is one read of a host's
 * GPU row from LDS, a count of its committed GPUs, one wave-wide minimum over a packed key and one
 * busy-until time written back. Runs that body `iters` times (1..2^24) in a dependent chain, one
 * wave per compute unit, on `stream` (a hipStream_t or NULL), twice, and returns the second pass's
 * nanoseconds per iteration in *ns_out (host memory). Synchronises the stream; allocates and frees
 * a few KB of device memory.
 * Errors: NBOS_E_ARG, NBOS_E_HIP, NBOS_E_NOMEM.
 */
int32_t nbos_chain_floor_ns(void *stream, int32_t iters, float *ns_out);

/* Free the handle and its device buffers (synchronises the stream). NULL is a no-op. */
void nbos_replay_destroy(nbos_replay *h);

/* Static, NUL-terminated description of a status code. */
const char *nbos_strerror(int32_t status);

/* After nbos_replay_create returned NBOS_E_HIP on this thread: the runtime call that failed and the
 * runtime's message for it, NUL-terminated, valid until the thread's next create. "" otherwise. */
const char *nbos_last_error_detail(void);

/* sizeof(nbos_stats) as compiled, for binding self-checks. */
int32_t nbos_sizeof_stats(void);

#ifdef __cplusplus
}
#endif
#endif /* NBOS_H */
