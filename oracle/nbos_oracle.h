/*
 * nbos_oracle.h — interface of the CPU oracle (TEST INFRASTRUCTURE, not product).
 *
 * A plain, single-threaded, eager discrete-event replay of NotebookOS's replica
 * placement and dynamic GPU-binding policy (paper Sections 3.2.1-3.2.3, 3.3,
 * 3.4.1, 3.4.2), written from the paper's description. It shares no code,
 * header or table with the GPU library; its own types are declared here.
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark call it.
 * All pointers are host pointers.
 */
#ifndef NBOS_ORACLE_H
#define NBOS_ORACLE_H
#include <stdint.h>

enum { ORC_EV_START = 0, ORC_EV_CELL = 1, ORC_EV_END = 2 };

enum {
  ORC_F_MIGRATE = 1, ORC_F_SCALE_OUT = 2, ORC_F_SCALE_IN = 4,
  ORC_F_AUTOSCALE = 0x20,   /* Section 3.4.2: periodic expected-capacity test f * sum C    */
  ORC_F_DYNAMIC_SR = 0x40,  /* Section 3.4.1: cluster-wide subscription ratio as the limit */
  ORC_F_STICKY = 0x80,      /* election variant: the previous executor leads again if it can */
  ORC_F_BATCH = 0x100,      /* replay the Batch baseline of the paper's "Baselines" section (orc_replay_batch)  */
  ORC_F_WARM_POOL = 0x200,  /* Section 3.2.3: pre-warmed containers shorten a migration        */
  ORC_F_CLOSED_LOOP = 0x400 /* a session's next event comes a think time after its previous
                               cell is over (not at its time in the trace)                    */
};

/* decision outcomes written to the log / folded into the digest */
enum {
  ORC_D_PLACE = 1, ORC_D_PLACE_NEW = 2, ORC_D_REJECT = 3, ORC_D_START = 4,
  ORC_D_MIGRATE = 5, ORC_D_SCALE_CELL = 6, ORC_D_ABORT = 7, ORC_D_SCALE_IN = 8,
  ORC_D_SCALE_AUTO = 9,  /* host added by the periodic auto-scaler (session field 0) */
  ORC_D_BATCH_START = 10,/* Batch baseline: GPUs allocated to the session's job on host */
  ORC_D_BATCH_HOST = 11, /* Batch baseline: host provisioned for the job at the queue's head */
  ORC_D_MIGRATE_WARM = 12/* migration into a pre-warmed container on the target host          */
};

/* error returns of orc_replay (0 = ok) */
enum {
  ORC_E_ARG = -1,        /* parameter out of range                                  */
  ORC_E_INPUT = -2,      /* trace invalid (unsorted, bad kind / id / duration / g)  */
  ORC_E_NOMEM = -5,
  ORC_E_INVARIANT = -100 /* -100 - k: self-check k failed (only with check != 0)    */
};

typedef struct {
  int32_t hosts_initial, hosts_max, gpus_per_host;
  uint32_t flags;
  int32_t migration_delay_ms, boot_delay_ms;
  int32_t retry_interval_ms, max_retries;
  int32_t scale_interval_ms, scale_in_idle_pct, min_hosts;
  int32_t cap_milli;            /* subscription-ratio cap x 1000 of this replay */
  int32_t check;                /* != 0: verify the invariants after every item */
  int32_t autoscale_f_milli;    /* f x 1000 of the expected capacity f * sum C (paper: 1050) */
  int32_t scaling_buffer_hosts; /* extra hosts kept on top of the expected capacity          */
  int32_t batch_start_delay_ms; /* Batch baseline: container start per job (GPUs already held) */
  int32_t warm_pool_per_host;   /* pre-warmed containers kept per host, 1..4 (ORC_F_WARM_POOL)  */
  int32_t warm_migration_delay_ms; /* migration delay into a pre-warmed container            */
  int32_t prewarm_delay_ms;     /* time to provision one pre-warmed container                */
} orc_params;

typedef struct {
  uint32_t n_decisions;
  uint32_t sessions_placed, sessions_rejected;
  uint32_t cells_total, cells_immediate, cells_started, cells_queued, cells_aborted;
  uint32_t cells_dropped_busy, cells_dropped_unplaced;
  uint32_t executor_reused, migrations;
  uint32_t scale_out_hosts, scale_in_hosts, peak_hosts;
  uint32_t migrations_warm;     /* migrations that found a pre-warmed container                */
  int32_t  max_delay_ms, t_end_ms;
  uint32_t delay_hist[32];
  int64_t  sum_delay_ms, sum_tct_ms;
  int64_t  gpu_ms_executed, gpu_ms_committed, gpu_ms_provisioned;
  int64_t  reservation_gpu_ms, sub_gpu_ms;
  int64_t  replica_ms;          /* integral over [0, t_end] of the number of placed replicas */
  uint64_t digest;
} orc_result;

/* optional dump of the final cluster state, for tests */
typedef struct {
  int32_t *host_state;     /* [hosts_max] 0 off, 1 booting, 2 ready                 */
  int32_t *host_committed; /* [hosts_max] C                                          */
  int32_t *host_subscribed;/* [hosts_max] S                                          */
  int32_t *host_nrep;      /* [hosts_max]                                            */
  int32_t *sess_state;     /* [n_sessions] 0 unplaced 1 idle 2 busy 3 rejected 4 ended */
  int32_t *sess_hosts;     /* [n_sessions*3]                                         */
} orc_final;

/*
 * Replay one trace on one simulated cluster.
 *   ev_time / ev_dur / ev_sk  n_events entries; ev_sk = session | kind << 24
 *   sess_gpus                 n_sessions GPU requests
 *   log                       optional: receives up to log_cap decision codes
 *   fin                       optional: final state (arrays owned by the caller)
 * Returns 0 or a negative error.
 */
int orc_replay(const orc_params *p,
               int64_t n_events, const int32_t *ev_time, const int32_t *ev_dur,
               const int32_t *ev_sk,
               int32_t n_sessions, const uint8_t *sess_gpus,
               orc_result *out, uint64_t *log, int64_t log_cap, orc_final *fin);

/*
 * Replay the same trace under the Batch baseline (the paper's "Baselines" section): every cell is a job of its
 * own, first come first served, a container per job. Same argument meaning as orc_replay; of the
 * flags only ORC_F_BATCH and ORC_F_SCALE_OUT are accepted. Fields of the result that only exist
 * with replicas (placement, migration, subscription, Reservation) stay 0; cells_queued counts the
 * jobs that waited for GPUs.
 */
int orc_replay_batch(const orc_params *p,
                     int64_t n_events, const int32_t *ev_time, const int32_t *ev_dur,
                     const int32_t *ev_sk,
                     int32_t n_sessions, const uint8_t *sess_gpus,
                     orc_result *out, uint64_t *log, int64_t log_cap);

int orc_sizeof_result(void);

/*
 * Billing model of the "Monetary Cost" section applied to one result, in integer micro-dollars (each amount
 * rounded down): the provider pays `price` per host-hour provisioned; users pay markup_pct / 100
 * times the provider's rate in proportion to the GPUs they use; a standby replica (placed, not
 * executing) pays standby_permille / 1000 of the marked-up host rate. The Reservation baseline
 * pays the marked-up rate for its reserved GPUs. The paper's values: markup 115, standby 125.
 */
typedef struct {
  int64_t provider_cost;        /* price * provisioned host-hours                            */
  int64_t usage_revenue;        /* executing replicas: g / G of the marked-up host rate      */
  int64_t standby_revenue;      /* replica-hours not executing                               */
  int64_t reservation_revenue;  /* what the Reservation baseline would bill                  */
} orc_bill;

void orc_billing(const orc_result *r, int gpus_per_host, int64_t price_micro_per_host_hour,
                 int markup_pct, int standby_permille, orc_bill *out);

#endif
