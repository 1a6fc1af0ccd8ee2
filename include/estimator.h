/*
 * Batched Estimator for prediction-pipeline configurations -- C ABI.
 *
 * The Estimator (arXiv 1812.01776, Section 4.2) is a discrete-event simulation that replays a
 * sample query trace through a pipeline DAG (Section 2) under one candidate configuration --
 * per stage a hardware type, a maximum batch size and a replica count (Section 4.1, "an
 * individual model configuration") -- and yields the latency of every query.  The planner
 * (Section 4.3, Algorithms 1 and 2) calls it for every candidate it considers and keeps a
 * candidate only if 99% of the latencies are within the SLO (Section 2), preferring the
 * cheapest (Section 6, cost model).  This library evaluates many candidates against the same
 * trace in one call, on one AMD MI355X GPU (gfx950).
 *
 * Queueing model (Section 2.1 "maximum batch size", Section 3 "centralized batched queueing
 * system", Section 4.2): each stage has one FIFO queue ordered by (time the query became ready
 * at the stage, query index).  Whenever a replica of the stage is idle and the queue is not
 * empty, the replica takes the first min(max batch, queue length) queries at once; the whole
 * batch completes together after the profiled latency of a batch of that actual size.  A stage
 * with several parents becomes ready for a query at the maximum of the parents' completion
 * times; a query whose visit-mask bit for a stage is clear passes through that stage in zero
 * time (Section 4.1, scale factor); end-to-end completion is the maximum over sink stages.
 * All times are integer microseconds and saturate at EST_HORIZON_US.
 *
 * Conventions for every function:
 *   - returns EST_OK (0) or a negative error code; never aborts, never throws;
 *   - the caller owns every buffer it passes; nothing is retained after return except by
 *     estimator_create, which deep-copies the DAG and the profiles;
 *   - outputs are untouched when an error is returned;
 *   - a handle must not be used by two threads at once.
 */
#ifndef ESTIMATOR_H
#define ESTIMATOR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EST_OK 0
#define EST_EINVAL (-1)       /* bad argument, malformed DAG / profile / trace / configuration      */
#define EST_ENOMEM (-2)       /* host or device allocation failed, or workspace too small           */
#define EST_EDEVICE (-3)      /* HIP runtime error; text in estimator_last_error                    */
#define EST_EUNSUPPORTED (-4) /* valid input the implementation cannot handle (see est limits)      */
#define EST_EINTERNAL (-5)    /* the simulation kernel reported an inconsistency                    */

#define EST_MAX_STAGES 32
#define EST_MAX_BATCH 64
#define EST_MAX_REPLICAS 64
#define EST_STATIC_SCRATCH_BYTES (64u << 20) /* fixed scratch of estimator_run_static_dev, per GPU           */
#define EST_MAX_MERGE_SOURCES 8 /* most distinct nearest visited ancestors feeding one stage        */
#define EST_HORIZON_US 0xFFFFFFFFu /* every computed time is min(true time, horizon)                */

typedef struct estimator estimator_t; /* opaque; immutable after estimator_create */

/* Pipeline DAG (Section 2): stages are numbered in a topological order. */
typedef struct {
    uint32_t n_stages;          /* S, 1..EST_MAX_STAGES                                              */
    const uint32_t *parent_off; /* [S+1] CSR offsets into parent_idx, parent_off[0] == 0             */
    const uint32_t *parent_idx; /* parents of each stage; every parent index < the child's index     */
} est_dag_t;

/* Model profiles (Section 4.1): latency of one replica as a function of hardware and batch size. */
typedef struct {
    uint32_t n_hw;                /* H >= 1 hardware types                                            */
    uint32_t max_batch;           /* Bmax, 1..EST_MAX_BATCH                                           */
    const uint32_t *lat_us;       /* [S][H][Bmax]; entry b-1 = latency of a batch of b queries, > 0   */
    const uint64_t *cost_uusd_hr; /* [S][H] price of one replica, micro-dollars per hour             */
} est_profiles_t;

/* Sample trace (Section 4.2). */
typedef struct {
    uint64_t n;                 /* number of queries, < 2^31                                          */
    const uint32_t *arrival_us; /* [n] arrival times, non-decreasing                                  */
    const uint32_t *visit_mask; /* [n] bit s set = the query visits stage s                           */
} est_trace_t;

/* One stage of one candidate configuration; a candidate is S consecutive entries. */
typedef struct {
    uint8_t hw;        /* < H                         */
    uint8_t batch;     /* maximum batch size, 1..Bmax */
    uint16_t replicas; /* 1..EST_MAX_REPLICAS         */
} est_stage_cfg_t;

/* Per-candidate results, each array [n_cfg]. */
typedef struct {
    uint32_t *p99_us;       /* nearest-rank P99: the ceil(0.99 n)-th smallest latency; 0 if n == 0   */
    uint32_t *miss_count;   /* number of queries with latency > slo_us                               */
    uint64_t *cost_uusd_hr; /* sum over stages of replicas x price                                   */
} est_result_t;

/* Timing of the most recent run, measured with HIP events on the run's stream. */
typedef struct {
    uint32_t n_launches;      /* launches of the simulation kernel                                    */
    uint32_t n_slots;         /* wavefronts (each with its own scratch) that shared the candidates    */
    float sim_ms;             /* duration of the simulation kernel (simulation + P99 selection)       */
    float prep_ms;            /* trace / configuration preprocessing kernels                          */
    uint64_t stage_visits;    /* sum over stages of queries visiting the stage (per candidate)        */
    uint64_t workspace_bytes; /* device scratch used                                                  */
    float capture_ms;         /* estimator_run_shared_dev: the launch that simulates the bases (part of sim_ms) */
    float ops_run_fraction;   /* estimator_run_shared_dev: operations run / (candidates x operations); else 0    */
    uint32_t waves_per_candidate; /* 1, or 2 or 4 when the call had so few candidates that each was given a workgroup */
    uint32_t reserved;
} est_stats_t;

/*
 * Build a handle for one pipeline and its profiles (host pointers; deep-copied to host and device).
 * Errors: EST_EINVAL for NULLs, S out of range, a parent index >= its child, duplicate parents,
 * H == 0, Bmax out of range, or any latency entry equal to 0; EST_EDEVICE if no usable GPU.
 */
int estimator_create(const est_dag_t *dag, const est_profiles_t *profiles, estimator_t **out);

/*
 * Simulate n_cfg candidates against one trace.  ALL POINTERS ARE HOST POINTERS; inputs are
 * copied to the GPU, results copied back; the call returns when the results are in place.
 * configs is [n_cfg][S].  n_cfg == 0 or trace->n == 0 succeeds (p99 = 0, miss_count = 0).
 * Errors: EST_EINVAL for NULLs, non-monotone arrivals, a configuration entry out of range, or a
 * trace whose last arrival + sum over stages of the largest profiled latency + slo_us reaches
 * the horizon; EST_EUNSUPPORTED if a stage would need more than EST_MAX_MERGE_SOURCES input
 * streams; EST_ENOMEM; EST_EDEVICE.
 */
int estimator_run(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs,
                  uint64_t n_cfg, uint32_t slo_us, est_result_t *out);

/*
 * The same with every array already in GPU memory: trace->arrival_us, trace->visit_mask,
 * configs and the three arrays of out are DEVICE pointers (the structs themselves live on the
 * host).  workspace is a device scratch buffer of workspace_bytes bytes owned by the caller, or
 * NULL to let the library allocate (and cache in the handle) what it needs; a smaller workspace
 * means fewer wavefronts share the candidates (scratch is per wavefront, not per candidate).  hip_stream is a hipStream_t
 * (NULL = the default stream); all work is enqueued on it and the call returns after that work
 * has completed.  Same errors as estimator_run; EST_ENOMEM if the workspace cannot hold one
 * candidate.
 */
int estimator_run_dev(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs,
                      uint64_t n_cfg, uint32_t slo_us, est_result_t *out, void *workspace,
                      uint64_t workspace_bytes, void *hip_stream);

/*
 * estimator_run_dev for callers that cannot allocate device memory (code that must not call hipMalloc:
 * tight serving loops, harnesses that forbid it): the scratch is a fixed array of
 * EST_STATIC_SCRATCH_BYTES bytes inside the library's device code, which every GPU the library runs on
 * holds until the process ends, and the call makes no hipMalloc, hipFree or other allocating call (the
 * events and the page-locked staging it needs were made by estimator_create).  Arguments, results and
 * errors as estimator_run_dev with that scratch; EST_ENOMEM, with the sizes in estimator_last_error,
 * when the fixed scratch cannot hold the run's per-query tables plus one candidate
 * (estimator_workspace_bytes(h, n, 1) says what a run needs at least).  All calls on one GPU share the
 * array, from any handle: calls that overlap in time on one GPU race.  Nothing is kept in it between calls.
 */
int estimator_run_static_dev(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs,
                             uint64_t n_cfg, uint32_t slo_us, est_result_t *out, void *hip_stream);

/*
 * Per-query latencies (Section 4.2: the Estimator returns the latency of each query), for
 * checking: lat_us_out is [n_cfg][n], host memory, indexed by query.  Host pointers throughout.
 */
int estimator_run_latencies(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs,
                            uint64_t n_cfg, uint32_t *lat_us_out);

/*
 * estimator_run_dev for candidates that share upstream stages with a base configuration, as the
 * candidates of one step of the planner's search do (Section 4.3: each action changes one model of the
 * current configuration).  A stage's completions depend only on the configuration of the stage and of
 * its ancestors in the pipeline, so for candidate i every stage that is configured, together with all
 * its ancestors, as in bases[base_of[i]] is simulated once for that base instead of once per
 * candidate.  Results are those of estimator_run_dev on configs, bit for bit; bases are not reported.
 * bases is [n_bases][S], configs [n_cfg][S], base_of [n_cfg] with entries < n_bases: DEVICE
 * pointers, like the trace arrays and the arrays of out.  A candidate may differ from its base in
 * any number of stages (sharing shrinks accordingly); n_bases == 0 behaves as estimator_run_dev.
 * The library allocates the scratch (cached in the handle like estimator_run_dev's).  The streams shared
 * by one base take 8 bytes x queries per shared stream; when those of all bases do not fit, the bases
 * are taken in rounds, the next round's bases running on a second stream of the library's own (default
 * priority) beside the current round's candidates; when the rounds the memory forces are estimated to take
 * longer than simulating every candidate on its own, the call does that instead (est_stats_t.ops_run_fraction
 * then reads 1; the environment variable EST_SHARED_ALWAYS switches this off, for measurements).  All work has
 * completed when the call returns.
 * Errors as estimator_run_dev; EST_EINVAL for a base_of entry out of range; EST_ENOMEM when not even
 * one base's streams fit beside one candidate's scratch; EST_EUNSUPPORTED for pipelines whose run
 * needs more than 64 operations or streams.
 */
int estimator_run_shared_dev(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *bases, uint64_t n_bases,
                             const est_stage_cfg_t *configs, const uint32_t *base_of, uint64_t n_cfg, uint32_t slo_us,
                             est_result_t *out, void *hip_stream);

/* Device-pointer variant of estimator_run_latencies; lat_us_out is a device buffer [n_cfg][n]. */
int estimator_run_latencies_dev(estimator_t *h, const est_trace_t *trace,
                                const est_stage_cfg_t *configs, uint64_t n_cfg, uint32_t *lat_us_out,
                                void *workspace, uint64_t workspace_bytes, void *hip_stream);

/*
 * Device scratch, in bytes, that gives every one of n_cfg candidates of an n-query trace its own
 * wavefront (an upper bound: it assumes every stage forks).  Smaller workspaces work, with fewer
 * wavefronts.  Returns 0 on a NULL handle.
 */
uint64_t estimator_workspace_bytes(const estimator_t *h, uint64_t n, uint64_t n_cfg);

/*
 * The greedy planner of Section 4.3 on top of the batched Estimator: Algorithm 1 (Initialize: batch 1,
 * one replica and the lowest-latency hardware everywhere; infeasible if the batch-1 service time of
 * the longest DAG path exceeds the SLO; otherwise add a replica to the throughput bottleneck until
 * the Estimator's P99 is within the SLO) followed by Algorithm 2 (MinimizeCost: repeatedly apply,
 * among IncreaseBatch (x2), RemoveReplica (-1) and DowngradeHW (next cheaper hardware, that model
 * re-initialised and locally re-optimised) on every model, the feasible result of lowest cost, until
 * no action has a feasible result).  Throughput of a stage = replicas x batch / latency(batch) /
 * fraction of the trace's queries that visit it.  Every feasibility test is one simulated candidate;
 * the candidates of one step are simulated together.
 */
#define EST_PLAN_INIT 0           /* est_plan_step_t.action: the configuration Initialize returned */
#define EST_PLAN_INCREASE_BATCH 1
#define EST_PLAN_REMOVE_REPLICA 2
#define EST_PLAN_DOWNGRADE_HW 3

typedef struct {
    uint32_t feasible;        /* 0: no configuration within the limits meets the SLO (config_out untouched) */
    uint32_t n_steps;         /* accepted steps, the initial configuration included (may exceed steps_cap)   */
    uint32_t estimator_calls; /* batched simulation calls made                                               */
    uint32_t p99_us;          /* P99 of the returned configuration                                           */
    uint64_t candidates;      /* configurations simulated in total                                           */
    uint64_t cost_uusd_hr;    /* cost of the returned configuration                                          */
} est_plan_result_t;

typedef struct {
    uint32_t action;       /* EST_PLAN_*                                   */
    int32_t stage;         /* the model the action was applied to, -1 for EST_PLAN_INIT */
    uint64_t cost_uusd_hr; /* cost of the configuration after the step     */
} est_plan_step_t;

/*
 * Plan one pipeline for one trace and SLO.  trace holds HOST pointers.  max_replicas (1..EST_MAX_REPLICAS)
 * bounds the replicas of a stage.  config_out is [S] and receives the plan; steps_out ([steps_cap],
 * may be NULL when steps_cap is 0) receives the accepted steps in order.  Returns EST_OK also when
 * no feasible configuration exists (result->feasible == 0).  Errors as for estimator_run.
 */
int estimator_plan(estimator_t *h, const est_trace_t *trace, uint32_t slo_us, uint32_t max_replicas,
                   est_stage_cfg_t *config_out, est_plan_result_t *result, est_plan_step_t *steps_out,
                   uint32_t steps_cap);

/*
 * What the planner hands to the high-frequency tuner (Section 5, "Initialization"): the traffic
 * envelope of the sample trace and, per model, the single-replica throughput mu_m and the
 * max-provisioning ratio rho_m of a configuration.
 *   Envelope: window widths dT_i = service_time_us * 2^i for i = 0, 1, ... while dT_i <= 60 s (at
 *   least dT_0); max_queries[i] = the largest number of arrivals in any half-open window
 *   [t, t + dT_i) over the trace; the maximum rate r_i is max_queries[i] / dT_i.
 *   mu_m  = batch / latency(hw, batch) queries per second  = mu_num / mu_den (mu_den in seconds x 10^6,
 *           i.e. mu_num = batch * 10^6, mu_den = latency in us).
 *   rho_m = lambda * s_m / (replicas * mu_m), lambda = n / (last arrival - first arrival), s_m = share
 *           of the queries that visit the model (the tuner's replica rule k_m = ceil(r s_m / (mu_m rho_m))
 *           gives back the planned replica count at r = lambda)  = rho_num / rho_den; when the trace
 *           spans no time (fewer than two queries, or all arrivals equal) there is no rate and rho_m is
 *           reported as 0 / 0: test rho_den before dividing.
 * All ratios are exact integer pairs.  trace and config ([S]) are HOST pointers.
 */
#define EST_MAX_WINDOWS 32
typedef struct {
    uint32_t n_windows;
    uint32_t reserved;
    uint64_t window_us[EST_MAX_WINDOWS];
    uint32_t max_queries[EST_MAX_WINDOWS];
    uint64_t mu_num[EST_MAX_STAGES], mu_den[EST_MAX_STAGES];
    uint64_t rho_num[EST_MAX_STAGES], rho_den[EST_MAX_STAGES];
} est_handoff_t;

/* Errors: EST_EINVAL for NULLs, service_time_us == 0, non-monotone arrivals or a configuration entry out of range. */
int estimator_tuner_handoff(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *config,
                            uint32_t service_time_us, est_handoff_t *out);

/*
 * Latency tables for models whose latency depends on the input (Section 8, the second limitation: measure the
 * latency distribution over the sample queries while profiling and give the Estimator its tail as the processing
 * time, which yields feasible but costlier plans).  samples_us is [n_entries][n_samples], HOST memory: n_samples
 * measured latencies (1..EST_MAX_PROFILE_SAMPLES) for each entry of est_profiles_t.lat_us, in that array's order
 * ([S][H][Bmax] flattened).  lat_us_out [n_entries], HOST memory, receives per entry
 *   EST_TAIL_PERCENTILE: the nearest-rank percentile: the k-th smallest sample, k = ceil(param x n_samples / 10000),
 *                        param in hundredths of a percent, 1..10000 (9900 = the 99th percentile);
 *   EST_TAIL_SIGMA:      the smallest integer >= mean + (param / 1000) x sigma, sigma the population standard
 *                        deviation of the samples, param 0..10000 (3000 = three standard deviations).
 * Exact integer arithmetic, no handle, no device work.  Errors: EST_EINVAL for NULLs, n_samples or param out of
 * range, an unknown mode, or a result that is 0 or does not fit 32 bits; EST_ENOMEM.  lat_us_out is untouched on error.
 */
#define EST_TAIL_PERCENTILE 0
#define EST_TAIL_SIGMA 1
#define EST_MAX_PROFILE_SAMPLES 65536
int estimator_profile_tail(const uint32_t *samples_us, uint64_t n_entries, uint32_t n_samples, uint32_t mode,
                           uint32_t param, uint32_t *lat_us_out);

/* Fill *out with the timing of the last successful run on this handle. */
int estimator_last_stats(const estimator_t *h, est_stats_t *out);

/* Text of the last error on this handle ("" if none); valid until the next call on the handle. */
const char *estimator_last_error(const estimator_t *h);

/* Free the handle and everything it owns; estimator_destroy(NULL) is a no-op. */
void estimator_destroy(estimator_t *h);

#ifdef __cplusplus
}
#endif
#endif /* ESTIMATOR_H */
